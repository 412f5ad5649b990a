// Mask-based MVDR beamforming (arXiv 2212.05271, Section 2.3, Eq. (6)-(9)) for gfx950.
//
//   cov    : Phi_k = sum_t gamma_target y y^H,  Phi_bg = sum_t (sum_{k != target} gamma_k) y y^H
//            (Eq. (6), (7); the common 1/T cancels in Eq. (8)), fp64 partial sums per chunk of frames.
//   solve  : per (segment, frequency): Phi_bg += delta * tr(Phi_bg)/D * I, G = Phi_bg^-1 Phi_k,
//            H = G / (Re tr G + eps): column r of H is the filter of Eq. (8) for reference channel r;
//            also the beamformed target and background powers of every candidate r.
//   ref    : per segment: the reference channel with the largest ratio of the two powers summed over
//            frequency (lowest index on ties), unless the caller fixed it.
//   apply  : X = h_ref^H y  (Eq. (9)).
//
// Everything up to the filter is fp64 (the solve amplifies errors of the covariances by the condition
// number of Phi_bg); the output is rounded to complex64 at the end.  Y is used as handed over, without
// normalisation.
#include "gss_internal.h"

#include "gss_device.h"

namespace {

// ----------------------------------------------------------------------------------------------
// Covariance accumulation for D <= 8.  Same tile machinery as the EM pass: a workgroup of kPassWaves
// wavefronts per (segment, frequency, chunk); per tile, lane = frame loads y and the two weights into the
// wavefront's LDS region, then lane = (frame group, channel i) accumulates the two weighted outer products
// (lane type i owns y_i conj(y_b) at circular channel distance 1..4 plus its share of the diagonal).  Output: part[sf][chunk][2][E] packed (0: target, 1: background).
// ----------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kWave * kPassWaves) void mvdr_cov_small(
    gss_yview yv, const float* __restrict__ gamma, const int32_t* __restrict__ T_len,
    const int32_t* __restrict__ target, double* __restrict__ part, uint32_t* __restrict__ status,
    int F, int Tmax, int K, int C, int tiles_per_chunk) {
  constexpr int E = D * D;
  // the two weights of a frame sit in the two padding entries at the end of its row of the y tile (three
  // workgroups per CU fit that way)
  constexpr int WS = kYStride;
  constexpr int kTileDoubles = kWave * kYStride;
  constexpr int kRedDoubles = kPassWaves * 64 * 2;
  constexpr int kLdsDoubles = kPassWaves * kTileDoubles > kRedDoubles ? kPassWaves * kTileDoubles : kRedDoubles;
  __shared__ __attribute__((aligned(16))) double lds[kLdsDoubles];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int chunk = blockIdx.x % C;
  const long sf = blockIdx.x / C;
  const int s = (int)(sf / F);
  const int f = (int)(sf % F);
  int T;
  const float2* __restrict__ Yrow = y_row(yv, T_len, s, f, D, Tmax, T);
  int tgt = target[s];
  if (tgt < 0 || tgt >= K) {                        // out of range: flagged, then clamped
    if (threadIdx.x == 0 && chunk == 0 && f == 0) atomicOr(status, GSS_STATUS_BAD_TARGET);
    tgt = tgt < 0 ? 0 : K - 1;
  }

  double* __restrict__ sY = lds + wave * kTileDoubles;
  double* __restrict__ sW = sY + kYTurned + 8;
  double acc[8][2];
#pragma unroll
  for (int n = 0; n < 8; ++n) { acc[n][0] = 0.0; acc[n][1] = 0.0; }
  const int tg = lane >> 3, eg = lane & 7;

  const float* __restrict__ grow = gamma + ((long)s * K * F + f) * Tmax;   // + k * F * Tmax + t
  const long gk = (long)F * Tmax;

  const int tile_lo = chunk * tiles_per_chunk;
  int tile_hi = tile_lo + tiles_per_chunk;
  const int tile_end = (T + kWave - 1) / kWave;
  tile_hi = tile_hi < tile_end ? tile_hi : tile_end;
  // One tile of 64 frames per step; the loads of the wavefront's next tile are issued before the arithmetic
  // of the current one.  A lane beyond T reads frame 0 (its weights are forced to zero).
  float2 yraw[D];
  float gv[GSS_MAX_K];
  auto load_tile = [&](int tile) {
    const int t = tile * kWave + lane;
    const long tc = t < T ? t : 0;
#pragma unroll
    for (int d = 0; d < D; ++d) yraw[d] = Yrow[tc * D + d];
#pragma unroll
    for (int k = 0; k < GSS_MAX_K; ++k) gv[k] = k < K ? grow[k * gk + tc] : 0.f;
  };
  int tile = tile_lo + wave;
  if (tile < tile_hi) load_tile(tile);
  for (; tile < tile_hi; tile += kPassWaves) {
    const bool valid = tile * kWave + lane < T;
    {
      double yr[D], yi[D];
#pragma unroll
      for (int d = 0; d < D; ++d) { yr[d] = (double)yraw[d].x; yi[d] = (double)yraw[d].y; }
      store_tile_row<D>(sY + lane * kYStride, yr, yi);
    }
    double wt = 0.0, wb = 0.0;
#pragma unroll
    for (int k = 0; k < GSS_MAX_K; ++k) {
      const double g = (double)gv[k];                // 0 for k >= K
      if (k == tgt) wt = g; else wb += g;
    }
    sW[lane * WS + 0] = valid ? wt : 0.0;
    sW[lane * WS + 1] = valid ? wb : 0.0;
    if (tile + kPassWaves < tile_hi) load_tile(tile + kPassWaves);
    wave_lds_sync();
    accumulate_tile<2, WS>(sY, sW, tg, eg, acc);
    wave_lds_sync();
  }
  double none[2] = {0.0, 0.0};
  reduce_and_store_partials<D, 2, false>(acc, none, sY, lds, part + (sf * C + chunk) * (long)(2 * E), nullptr, lane, wave);
}

// ----------------------------------------------------------------------------------------------
// Solve for D <= 8: one wavefront per (segment, frequency), lane (i, j) = (l / D, l % D).
// Outputs: H[sf][r][d] (complex fp64, filter for reference r, channel d) and pw[sf][r][2] =
// (Re h_r^H Phi_k h_r, Re h_r^H Phi_bg' h_r) with Phi_bg' the loaded background covariance.
// ----------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kWave) void mvdr_solve_small(
    const double* __restrict__ part, double2* __restrict__ H, double* __restrict__ pw,
    uint32_t* __restrict__ status, int C) {
  constexpr int E = D * D;
  __shared__ double sR[2][E];
  __shared__ double sKr[D][D], sKi[D][D];      // Phi_k
  __shared__ double sBr[D][D], sBi[D][D];      // loaded Phi_bg (kept for the power terms)
  __shared__ double sMr[D][D], sMi[D][D];      // working copy -> inverse
  __shared__ double sGr[D][D], sGi[D][D];      // G, then H

  const long sf = blockIdx.x;
  const int l = threadIdx.x;
  const bool on = l < E;
  const int i = l / D, j = l % D;

  if (on) {
    double a = 0.0, b = 0.0;
    for (int c = 0; c < C; ++c) {
      a += part[((sf * C + c) * 2 + 0) * (long)E + l];
      b += part[((sf * C + c) * 2 + 1) * (long)E + l];
    }
    sR[0][l] = a;
    sR[1][l] = b;
  }
  __syncthreads();
  double trb = 0.0, trk = 0.0;
#pragma unroll
  for (int r = 0; r < D; ++r) {
    trb += sR[1][gss_packed_row(r, D)];
    trk += sR[0][gss_packed_row(r, D)];
  }
  if (!(trb > 0.0)) {
    // No background energy at all (an empty segment, or all-zero input): the filter is defined as zero.
    // With target energy but no background Eq. (8) has no solution; that case is flagged.
    if (trk > 0.0 && l == 0) atomicOr(status, GSS_STATUS_NONPD_PHI);
    if (on) H[(sf * D + j) * D + i] = make_double2(0.0, 0.0);
    if (l < D) { pw[(sf * D + l) * 2 + 0] = 0.0; pw[(sf * D + l) * 2 + 1] = 0.0; }
    return;
  }
  if (on) {
    double kr, ki = 0.0, br, bi = 0.0;
    if (i == j) {
      kr = sR[0][gss_packed_row(i, D)];
      br = sR[1][gss_packed_row(i, D)] + GSS_DELTA_BF * trb / (double)D;
    } else {
      const int lo = i < j ? i : j, hi = i < j ? j : i;
      const int p = gss_packed_row(lo, D) + 1 + 2 * (hi - lo - 1);
      kr = sR[0][p]; ki = sR[0][p + 1];
      br = sR[1][p]; bi = sR[1][p + 1];
      if (i > j) { ki = -ki; bi = -bi; }
    }
    sKr[i][j] = kr; sKi[i][j] = ki;
    sBr[i][j] = br; sBi[i][j] = bi;
    sMr[i][j] = br; sMi[i][j] = bi;
  }
  __syncthreads();
  // in-place Gauss-Jordan inversion of the Hermitian positive-definite loaded Phi_bg
  for (int p = 0; p < D; ++p) {
    double piv = sMr[p][p];
    if (!(piv > 1e-300)) {
      piv = 1e-300;
      if (l == 0) atomicOr(status, GSS_STATUS_NONPD_PHI);
    }
    const double rp = 1.0 / piv;
    double nr = 0.0, ni = 0.0;
    if (on) {
      const double air = sMr[i][p], aii = sMi[i][p];
      const double apr = sMr[p][j], api = sMi[p][j];
      if (i == p && j == p) {
        nr = rp;
      } else if (i == p) {
        nr = apr * rp; ni = api * rp;
      } else if (j == p) {
        nr = -air * rp; ni = -aii * rp;
      } else {
        nr = sMr[i][j] - (air * apr - aii * api) * rp;
        ni = sMi[i][j] - (air * api + aii * apr) * rp;
      }
    }
    __syncthreads();
    if (on) { sMr[i][j] = nr; sMi[i][j] = ni; }
    __syncthreads();
  }
  // G = Phi_bg^-1 Phi_k
  if (on) {
    double gr = 0.0, gi = 0.0;
#pragma unroll
    for (int m = 0; m < D; ++m) {
      const double ar = sMr[i][m], ai = sMi[i][m], br = sKr[m][j], bi = sKi[m][j];
      gr += ar * br - ai * bi;
      gi += ar * bi + ai * br;
    }
    sGr[i][j] = gr; sGi[i][j] = gi;
  }
  __syncthreads();
  double tr = 0.0;
#pragma unroll
  for (int r = 0; r < D; ++r) tr += sGr[r][r];
  const double inv = 1.0 / (tr + GSS_EPS_TRACE);
  if (on) {
    const double hr = sGr[i][j] * inv, hi = sGi[i][j] * inv;   // H[d = i][r = j]
    H[(sf * D + j) * D + i] = make_double2(hr, hi);
    sGr[i][j] = hr; sGi[i][j] = hi;
  }
  __syncthreads();
  // powers of candidate r: h_r^H Phi h_r, lanes l < D handle r = l
  if (l < D) {
    const int r = l;
    double pk = 0.0, pb = 0.0;
    for (int a = 0; a < D; ++a) {
      double tkr = 0.0, tki = 0.0, tbr = 0.0, tbi = 0.0;       // (Phi h_r)[a]
      for (int b = 0; b < D; ++b) {
        const double hr = sGr[b][r], hi = sGi[b][r];
        tkr += sKr[a][b] * hr - sKi[a][b] * hi;  tki += sKr[a][b] * hi + sKi[a][b] * hr;
        tbr += sBr[a][b] * hr - sBi[a][b] * hi;  tbi += sBr[a][b] * hi + sBi[a][b] * hr;
      }
      const double hr = sGr[a][r], hi = sGi[a][r];
      pk += hr * tkr + hi * tki;                               // Re(conj(h_a) * t_a)
      pb += hr * tbr + hi * tbi;
    }
    pw[(sf * D + r) * 2 + 0] = pk;
    pw[(sf * D + r) * 2 + 1] = pb;
  }
}

// ----------------------------------------------------------------------------------------------
// Reference channel per segment: one workgroup of 1024 threads per segment; thread (r, j) sums candidate
// r's powers over the frequencies f = j, j + 32, ..., the 32 partial sums per candidate are added in a
// fixed order (deterministic), then thread 0 takes the arg-max (lowest index on ties).
// 0 <= ref_io[s] < D on entry is kept; a value >= D is flagged in the status word and replaced by the choice.
// ----------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void mvdr_ref(const double* __restrict__ pw, int32_t* __restrict__ ref_io,
                                                 uint32_t* __restrict__ status, int F, int D) {
  __shared__ double snum[32][33], sden[32][33];
  __shared__ double score[GSS_MAX_D];
  const int s = blockIdx.x;
  const int r = threadIdx.x & 31, j = threadIdx.x >> 5;
  double num = 0.0, den = 0.0;
  if (r < D) {
    for (int f = j; f < F; f += 32) {
      num += pw[(((long)s * F + f) * D + r) * 2 + 0];
      den += pw[(((long)s * F + f) * D + r) * 2 + 1];
    }
  }
  snum[r][j] = num;
  sden[r][j] = den;
  __syncthreads();
  if (j == 0 && r < D) {
    double n = 0.0, d = 0.0;
    for (int q = 0; q < 32; ++q) { n += snum[r][q]; d += sden[r][q]; }
    score[r] = n / fmax(d, GSS_EPS_SNR);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int cur = ref_io[s];
    if (cur >= D) atomicOr(status, GSS_STATUS_BAD_REF);
    if (cur < 0 || cur >= D) {
      int best = 0;
      for (int c = 1; c < D; ++c)
        if (score[c] > score[best]) best = c;
      cur = best;
    }
    ref_io[s] = cur;
  }
}

// Reference channel per (segment, frequency): the candidate with the largest ratio of the two powers at that
// frequency alone (lowest index on ties); 0 <= ref_io[sf] < D on entry is kept.  One thread per (s, f).
__global__ __launch_bounds__(256) void mvdr_ref_freq(const double* __restrict__ pw, int32_t* __restrict__ ref_io,
                                                     uint32_t* __restrict__ status, long n_sf, int D) {
  const long sf = blockIdx.x * (long)blockDim.x + threadIdx.x;
  if (sf >= n_sf) return;
  int cur = ref_io[sf];
  if (cur >= D) atomicOr(status, GSS_STATUS_BAD_REF);
  if (cur < 0 || cur >= D) {
    int best = 0;
    double best_score = pw[(sf * D + 0) * 2 + 0] / fmax(pw[(sf * D + 0) * 2 + 1], GSS_EPS_SNR);
    for (int c = 1; c < D; ++c) {
      const double sc = pw[(sf * D + c) * 2 + 0] / fmax(pw[(sf * D + c) * 2 + 1], GSS_EPS_SNR);
      if (sc > best_score) { best = c; best_score = sc; }
    }
    cur = best;
  }
  ref_io[sf] = cur;
}

// ----------------------------------------------------------------------------------------------
// Apply: X[s][f][t] = sum_d conj(h[d]) y[t][d], lane = frame; the filter is wave-uniform.
// Grid: blockIdx.x = chunk + C * (f + F * s), 256 frames per workgroup step.
// ----------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void mvdr_apply_small(
    gss_yview yv, const double2* __restrict__ H, const int32_t* __restrict__ ref,
    const int32_t* __restrict__ T_len, float2* __restrict__ X, int F, int Tmax, int C, int frames_per_chunk,
    int ref_per_f) {
  const int chunk = blockIdx.x % C;
  const long sf = blockIdx.x / C;
  const int s = (int)(sf / F);
  int T;
  const float2* __restrict__ Yrow = y_row(yv, T_len, s, (int)(sf % F), D, Tmax, T);
  int r = ref[ref_per_f ? sf : (long)s];
  r = r < 0 ? 0 : (r >= D ? D - 1 : r);
  double hr[D], hi[D];
#pragma unroll
  for (int d = 0; d < D; ++d) {
    const double2 h = H[(sf * D + r) * D + d];
    hr[d] = h.x;
    hi[d] = h.y;
  }
  float2* __restrict__ Xrow = X + sf * (long)Tmax;
  const int t_lo = chunk * frames_per_chunk;
  int t_hi = t_lo + frames_per_chunk;
  t_hi = t_hi < Tmax ? t_hi : Tmax;
  for (int t = t_lo + threadIdx.x; t < t_hi; t += blockDim.x) {
    double xr = 0.0, xi = 0.0;
    if (t < T) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        const float2 v = Yrow[(long)t * D + d];
        xr += hr[d] * (double)v.x + hi[d] * (double)v.y;     // conj(h) * y
        xi += hr[d] * (double)v.y - hi[d] * (double)v.x;
      }
    }
    Xrow[t] = make_float2((float)xr, (float)xi);
  }
}

template <int D>
int run_mvdr_small(gss_ctx* ctx, const gss_yview& Y, const float* gamma, const int32_t* T_len, int S, int F, int Tmax,
                   int K, const int32_t* target, int32_t* ref, int ref_per_f, float2* X, hipStream_t st) {
  const long n_sf = (long)S * F;
  constexpr int E = D * D;
  const int tiles = (Tmax + kWave - 1) / kWave;
  // Chunks per problem: as many as fit the resident workgroup slots in one round (the wavefronts of a
  // workgroup take the chunk's tiles round-robin, so a chunk may hold any number of tiles).
  static const int wgs_per_cu = resident_wgs(mvdr_cov_small<D>, kWave * kPassWaves, 2);
  long c_target = ((long)ctx->num_cu * wgs_per_cu) / n_sf;
  if (c_target < 1) c_target = 1;
  if (c_target > tiles) c_target = tiles;
  const int tpc = (int)((tiles + c_target - 1) / c_target);
  const int C = (tiles + tpc - 1) / tpc;
  if (n_sf * C > 0x7fffffffL) return GSS_EUNSUPPORTED;

  size_t o = 0;
  const size_t off_part = o; o = gss_align_up(o + (size_t)n_sf * C * 2 * E * sizeof(double), 256);
  const size_t off_H = o;    o = gss_align_up(o + (size_t)n_sf * E * sizeof(double2), 256);
  const size_t off_pw = o;   o = gss_align_up(o + (size_t)n_sf * D * 2 * sizeof(double), 256);
  int rc = gss_ensure_scratch(ctx, o);
  if (rc != GSS_OK) return rc;
  char* base = (char*)ctx->scratch;
  double* part = (double*)(base + off_part);
  double2* H = (double2*)(base + off_H);
  double* pw = (double*)(base + off_pw);

  hipLaunchKernelGGL((mvdr_cov_small<D>), dim3((unsigned)(n_sf * C)), dim3(kWave * kPassWaves), 0, st, Y, gamma, T_len,
                     target, part, ctx->status, F, Tmax, K, C, tpc);
  hipLaunchKernelGGL((mvdr_solve_small<D>), dim3((unsigned)n_sf), dim3(kWave), 0, st, part, H, pw, ctx->status, C);
  gss_launch_mvdr_ref(pw, ref, ctx->status, S, F, D, ref_per_f, st);
  const int fpc = 1024;
  const int CA = (Tmax + fpc - 1) / fpc;
  if (n_sf * CA > 0x7fffffffL) return GSS_EUNSUPPORTED;
  hipLaunchKernelGGL((mvdr_apply_small<D>), dim3((unsigned)(n_sf * CA)), dim3(256), 0, st, Y, H, ref, T_len, X, F, Tmax,
                     CA, fpc, ref_per_f);
  if (hipGetLastError() != hipSuccess) return GSS_EHIP;
  return GSS_OK;
}

}  // namespace

void gss_launch_mvdr_ref(const double* pw, int32_t* ref, uint32_t* status, int S, int F, int D, int ref_per_f,
                         hipStream_t st) {
  if (ref_per_f) {
    const long n_sf = (long)S * F;
    hipLaunchKernelGGL(mvdr_ref_freq, dim3((unsigned)((n_sf + 255) / 256)), dim3(256), 0, st, pw, ref, status, n_sf, D);
    return;
  }
  hipLaunchKernelGGL(mvdr_ref, dim3((unsigned)S), dim3(1024), 0, st, pw, ref, status, F, D);
}

static int mvdr_dispatch(gss_ctx* ctx, const gss_yview& yv, const float* gamma, const int32_t* T_len, int S, int F,
                         int Tmax, int D, int K, const int32_t* target, int32_t* ref, int ref_mode, float* X,
                         void* stream) {
  if (S <= 0 || F <= 0 || Tmax <= 0 || D <= 0 || K <= 0) return GSS_EINVAL;
  if (ref_mode != GSS_REF_PER_SEGMENT && ref_mode != GSS_REF_PER_FREQUENCY) return GSS_EINVAL;
  if (D > GSS_MAX_D || K > GSS_MAX_K) return GSS_EUNSUPPORTED;
  if (hipSetDevice(ctx->device) != hipSuccess) return GSS_EHIP;
  hipStream_t st = (hipStream_t)stream;
  float2* Xc = (float2*)X;
  const int per_f = ref_mode == GSS_REF_PER_FREQUENCY;
  switch (D) {
#define GSS_CASE_D(DD) \
  case DD: return run_mvdr_small<DD>(ctx, yv, gamma, T_len, S, F, Tmax, K, target, ref, per_f, Xc, st);
    GSS_CASE_D(1) GSS_CASE_D(2) GSS_CASE_D(3) GSS_CASE_D(4) GSS_CASE_D(5) GSS_CASE_D(6) GSS_CASE_D(7) GSS_CASE_D(8)
#undef GSS_CASE_D
    default: return gss_mvdr_large(ctx, yv, gamma, T_len, S, F, Tmax, D, K, target, ref, per_f, X, st);
  }
}

extern "C" int gss_mvdr(gss_ctx* ctx, const float* Y, const float* gamma, const int32_t* T_len,
                        int S, int F, int Tmax, int D, int K, const int32_t* target, int32_t* ref,
                        float* X, void* stream) {
  return gss_mvdr_ex(ctx, Y, 0, nullptr, gamma, T_len, S, F, Tmax, D, K, target, GSS_REF_PER_SEGMENT, ref, X, stream);
}

extern "C" int gss_mvdr_frames(gss_ctx* ctx, const float* Yrec, int64_t Trec, const int64_t* frame0, const float* gamma,
                               const int32_t* T_len, int S, int F, int Tmax, int D, int K, const int32_t* target,
                               int32_t* ref, float* X, void* stream) {
  if (!frame0 || Trec <= 0) return GSS_EINVAL;
  return gss_mvdr_ex(ctx, Yrec, Trec, frame0, gamma, T_len, S, F, Tmax, D, K, target, GSS_REF_PER_SEGMENT, ref, X,
                     stream);
}

extern "C" int gss_mvdr_ex(gss_ctx* ctx, const float* Y, int64_t Trec, const int64_t* frame0, const float* gamma,
                           const int32_t* T_len, int S, int F, int Tmax, int D, int K, const int32_t* target,
                           int ref_mode, int32_t* ref, float* X, void* stream) {
  if (!ctx || !Y || !gamma || !target || !ref || !X) return GSS_EINVAL;
  if (F <= 0 || Tmax <= 0 || D <= 0 || Trec < 0) return GSS_EINVAL;
  if ((frame0 != nullptr) != (Trec > 0)) return GSS_EINVAL;
  const gss_yview yv = frame0 ? gss_frames_view(Y, Trec, frame0, D) : gss_dense_view(Y, F, Tmax, D);
  return mvdr_dispatch(ctx, yv, gamma, T_len, S, F, Tmax, D, K, target, ref, ref_mode, X, stream);
}
