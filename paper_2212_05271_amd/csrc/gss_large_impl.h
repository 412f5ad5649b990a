// EM and MVDR kernels for large arrays, 9 <= D <= 32 channels (e.g. multi-array set-ups with 24
// microphones).  Same algorithm, same fp64 arithmetic and the same pass / factor structure as the D <= 8
// kernels (arXiv 2212.05271, Section 2.2 and 2.3); what changes is the mapping:
//
//   * D is a run-time value; the Hermitian outer product has M = D (D + 1) / 2 "items" (i <= j), each a
//     real diagonal entry or a complex off-diagonal one.  Coefficients are class-major, coef[sf][k][CP]
//     (entries 2 m and 2 m + 1 multiply Re and Im of item m; CP = 2 M rounded up to whole groups of 16,
//     zero padding); partial sums are item-major, part[workgroup][m][k][2].
//   * The frames of a tile sit in LDS as fp32 (exactly as they came), because D * 16 bytes of fp64 per
//     frame would not leave room for two workgroups per compute unit.
//   * Phase 1 (lane = frame) walks the items 8 at a time in a run-time loop, reading y_i, y_j of its own
//     frame from LDS; the 16 coefficients of a group sit in one register pair per class and reach the FMAs
//     through the row-broadcast operand selector.
//   * Phase 2 (lane = a few items, frames in sequence): each lane owns NR items m = lane, lane + 64, ...,
//     forms them for every frame of the tile from LDS and accumulates K weighted sums per real part.
//   * Classes that are inactive in all 64 frames of a tile are skipped in both phases.
#pragma once

#include "gss_internal.h"

#include "gss_device.h"

namespace {

constexpr int kLargeWaves = 4;

__host__ __device__ inline int item_index(int i, int j, int D) { return i * D - i * (i - 1) / 2 + (j - i); }   // i <= j
__host__ __device__ inline int num_items(int D) { return D * (D + 1) / 2; }

// (i, j) of item m, by walking the rows (run once per lane and item at kernel start).
__device__ __forceinline__ void item_ij(int m, int D, int& i, int& j) {
  int r = 0, left = m;
  while (left >= D - r) { left -= D - r; ++r; }
  i = r;
  j = r + left;
}

__device__ __forceinline__ double ipow_rt(double x, int n) {   // x^n, n >= 1
  double r = 1.0, b = x;
  while (n) {
    if (n & 1) r *= b;
    b *= b;
    n >>= 1;
  }
  return r;
}

// Coefficient layout for 9 <= D <= 32: class-major, coef[sf][k][CP], in groups of 16 doubles = (Re, Im) of 8 items.
// The items (i, j), i <= j, of row i fill ceil((D - i) / 8) groups of their own, in the order of j; the last group
// of a row is padded (the padding is zero and never used).  A group never spans two rows, so the pass kernel
// walks a group with one y_i and consecutive y_j.
__host__ __device__ inline int groups_of_lengths_up_to(int n) {      // sum over L = 1 .. n of ceil(L / 8)
  const int q = n >> 3, r = n & 7;
  return 4 * q * (q + 1) + r * (q + 1);
}
__host__ __device__ inline int coef_groups(int D) { return groups_of_lengths_up_to(D); }
__host__ __device__ inline int coef_pitch(int D) { return 16 * coef_groups(D); }
// first group of row i (rows 0 .. i - 1 have the lengths D, D - 1, ..., D - i + 1)
__host__ __device__ inline int row_group(int i, int D) { return groups_of_lengths_up_to(D) - groups_of_lengths_up_to(D - i); }
// position (in doubles) of the Re coefficient of item (i, j), i <= j; Im follows
__host__ __device__ inline int coef_pos(int i, int j, int D) {
  return 16 * (row_group(i, D) + ((j - i) >> 3)) + 2 * ((j - i) & 7);
}

__global__ void em_init_coef_large(double* __restrict__ coef, double* __restrict__ cmant, int32_t* __restrict__ cexp,
                                   int D, int K, long n_sf) {
  const int CP = coef_pitch(D);
  const long total = n_sf * K * CP;
  for (long x = blockIdx.x * (long)blockDim.x + threadIdx.x; x < total; x += (long)gridDim.x * blockDim.x) {
    const int c = (int)(x % CP);
    double v = 0.0;
    if ((c & 15) == 0) {                     // first entry of a group: 1 if the group opens a row (the diagonal item)
      int g = c >> 4, r = 0;
      while (r < D && g >= (D - r + 7) / 8) { g -= (D - r + 7) / 8; ++r; }
      v = (r < D && g == 0) ? 1.0 : 0.0;
    }
    coef[x] = v;
  }
  const long nl = n_sf * K;
  for (long x = blockIdx.x * (long)blockDim.x + threadIdx.x; x < nl; x += (long)gridDim.x * blockDim.x) {
    cmant[x] = 0.5;
    cexp[x] = 1;
  }
}

// Cooperative, coalesced copy of one tile of frames [t0, t0 + 64) of a (segment, frequency) row into the
// wavefront's LDS tile sY[frame][D] (float2, row stride RS float2); frames at or beyond T become zero.
// The tile is one contiguous run of 64 D values in memory; lane l copies values l, l + 64, ... (D of them).  Their
// frame and channel are stepped without divisions, and the loads go out six at a time before the first of them
// is stored (one at a time, every value would wait out a full memory latency).
__device__ __forceinline__ void load_tile(const float2* __restrict__ Yrow, int t0, int T, int D, int RS,
                                          float2* __restrict__ sY, int lane) {
  constexpr int kBatch = 12;
  const int rstep = kWave / D, cstep = kWave % D;          // frame and channel advance per 64 values
  int r = lane / D, c = lane - r * D;
  const float2* __restrict__ src = Yrow + (long)t0 * D + lane;
  const int rows = T - t0;                                   // frames of the tile that exist (may exceed 64)
  for (int i0 = 0; i0 < D; i0 += kBatch) {
    float2 v[kBatch];
    int off[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      v[u] = make_float2(0.f, 0.f);
      off[u] = r * RS + c;
      if (i0 + u < D) {
        if (r < rows) v[u] = src[(long)(i0 + u) * kWave];
        c += cstep;
        r += rstep;
        if (c >= D) { c -= D; ++r; }
      }
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u)
      if (i0 + u < D) sY[off[u]] = v[u];
  }
}

// Phase 2 for the lane's NR items over the 64 frames of the tile, for the classes of `mask` (wave-uniform; the
// weights of the other classes are zero in every frame of the tile).
template <int KW, int NR>
__device__ __forceinline__ void accumulate_items(const float2* __restrict__ sY, const double* __restrict__ sW, int RS,
                                                 int WS, const int (&oi)[NR], const int (&oj)[NR], unsigned mask,
                                                 double (&acc)[NR][2][KW]) {
#pragma unroll 1
  for (int r = 0; r < kWave; ++r) {
    double w[KW];
#pragma unroll
    for (int k = 0; k < KW; ++k) w[k] = sW[r * WS + k];
    double re[NR], im[NR];
#pragma unroll
    for (int n = 0; n < NR; ++n) {
      const float2 a = sY[r * RS + oi[n]];
      const float2 b = sY[r * RS + oj[n]];
      const double ar = a.x, ai = a.y, br = b.x, bi = b.y;
      re[n] = ar * br + ai * bi;          // Re(y_i conj(y_j)); |y_i|^2 on the diagonal
      im[n] = ai * br - ar * bi;          // Im(y_i conj(y_j)); 0 on the diagonal
    }
    static_for<0, KW>([&](auto KI) {
      constexpr int k = KI.value;
      if (class_on(mask, k)) {
#pragma unroll
        for (int n = 0; n < NR; ++n) {
          acc[n][0][k] = fma(w[k], re[n], acc[n][0][k]);
          acc[n][1][k] = fma(w[k], im[n], acc[n][1][k]);
        }
      }
    });
  }
}

// Sums the accumulators of the workgroup's wavefronts through LDS and writes out[m][k][2].
template <int KW, int NR>
__device__ __forceinline__ void reduce_items(double (&acc)[NR][2][KW], double* __restrict__ red, double* __restrict__ out,
                                             int M, int lane, int wave) {
  __syncthreads();
  for (int w = 0; w < kLargeWaves; ++w) {
    if (wave == w) {
#pragma unroll
      for (int n = 0; n < NR; ++n) {
        const int m = lane + kWave * n;
        if (m < M) {
#pragma unroll
          for (int k = 0; k < KW; ++k)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
              double* dst = &red[((long)m * KW + k) * 2 + p];
              *dst = (w == 0) ? acc[n][p][k] : *dst + acc[n][p][k];
            }
        }
      }
    }
    __syncthreads();
  }
  const int total = M * KW * 2;
  for (int x = threadIdx.x; x < total; x += kWave * kLargeWaves) out[x] = red[x];
}

// ----------------------------------------------------------------------------------------------
// EM pass, 9 <= D <= 32.  Grid: blockIdx.x = chunk + C * (f + F * s); the chunk's tiles are dealt to the
// wavefronts round-robin.  Dynamic LDS: kLargeWaves * (64 * RS float2 + 64 * WS doubles), reused for the
// final reduction (needs M * K * 2 doubles).
//
// Phase 1 (lane = frame) walks the items 8 at a time.  The 16 class coefficients of such a group (Re and Im
// of 8 items) sit in one register pair, entry lane mod 16 in every lane, fetched from memory one group ahead
// (a coalesced 128-byte read that the four rows of the wavefront share); the FMAs take them through the
// row-broadcast selector of the fp64 FMA.  Classes outside the tile's activity mask are skipped.
// ----------------------------------------------------------------------------------------------
// Wavefronts per SIMD that the register allocation of the pass kernel is held to: two where the 4 K NR registers
// of the phase-2 accumulators leave room for most of the rest within 256 (some values then go to scratch memory,
// which costs far less than the second wavefront brings: 20 to 36 % less time at 25 to 32 channels or 6 to 8
// classes), one otherwise (beyond 180 accumulator registers the spills reach the inner loops and the kernel gets
// two to three times slower than with one wavefront).
constexpr int pass_waves_per_simd(int K, int NR) { return 4 * K * NR <= 180 ? 2 : 1; }

template <int K, int NR, bool FINAL>
__global__ __launch_bounds__(kWave * kLargeWaves, pass_waves_per_simd(K, NR)) void em_pass_large(
    gss_yview yv, const uint8_t* __restrict__ abyte, const uint32_t* __restrict__ tmask,
    const int32_t* __restrict__ T_len,
    const double* __restrict__ coef, const double* __restrict__ cmant, const int32_t* __restrict__ cexp,
    double* __restrict__ part, double* __restrict__ npart, float* __restrict__ gamma, uint32_t* __restrict__ status,
    int F, int Tmax, int D, ChunkMap cmap, int RS, int tile_bytes) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  constexpr int WS = K | 1;
  const int M = num_items(D);
  const int CP = coef_pitch(D);
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  long sf;
  int chunk, tiles_per_chunk;
  chunk_decode(cmap, blockIdx.x, sf, chunk, tiles_per_chunk);
  const int s = (int)(sf / F);
  const int f = (int)(sf % F);
  int T;
  const float2* __restrict__ Yrow = y_row(yv, T_len, s, f, D, Tmax, T);
  const int t_end = FINAL ? Tmax : T;

  float2* __restrict__ sY = reinterpret_cast<float2*>(lds_raw + (size_t)wave * tile_bytes);
  double* __restrict__ sW = reinterpret_cast<double*>(lds_raw + (size_t)wave * tile_bytes + (size_t)kWave * RS * sizeof(float2));

  const double* __restrict__ cf = coef + sf * (long)K * CP + (lane & 15);   // + k * CP + 16 * group
  const double* __restrict__ cm = cmant + sf * K;
  const int32_t* __restrict__ ce = cexp + sf * K;
  const uint8_t* __restrict__ abrow = abyte + (long)s * Tmax;
  const int tiles_total = (Tmax + kWave - 1) / kWave;
  typedef const __attribute__((address_space(4))) uint32_t* mask_ptr_t;
  const mask_ptr_t tmrow = (mask_ptr_t)(uintptr_t)(tmask + (long)s * tiles_total);

  int oi[NR], oj[NR];
  double acc[NR][2][K];
#pragma unroll
  for (int n = 0; n < NR; ++n) {
    int m = lane + kWave * n;
    if (m >= M) m = 0;                       // idle slot: computes item 0, never written out
    item_ij(m, D, oi[n], oj[n]);
#pragma unroll
    for (int k = 0; k < K; ++k) { acc[n][0][k] = 0.0; acc[n][1][k] = 0.0; }
  }
  double nacc[K];
#pragma unroll
  for (int k = 0; k < K; ++k) nacc[k] = 0.0;

  const int groups = coef_groups(D);
  const int tile_lo = chunk * tiles_per_chunk;
  int tile_hi = tile_lo + tiles_per_chunk;
  const int tile_end = (t_end + kWave - 1) / kWave;
  tile_hi = tile_hi < tile_end ? tile_hi : tile_end;
  for (int tile = tile_lo + wave; tile < tile_hi; tile += kLargeWaves) {
    const int t0 = tile * kWave;
    const int t = t0 + lane;
    const bool valid = t < T;
    const unsigned mask = tmrow[tile] & ((1u << K) - 1u);
    if constexpr (FINAL) {
      static_for<0, K>([&](auto KI) {
        constexpr int k = KI.value;
        if (!class_on(mask, k)) {
          if (t < Tmax) gamma[(((long)s * K + k) * F + f) * Tmax + t] = 0.f;
        }
      });
    }
    if (mask == 0u) continue;                // no frame of the tile has an active class
    load_tile(Yrow, t0, T, D, RS, sY, lane);
    unsigned abits = abrow[valid ? t : 0];
    abits = valid ? abits : 0u;
    wave_lds_sync();

    // ---- phase 1: q_k = <coef_k, y y^H> for the lane's frame ----
    double q[K][2];
#pragma unroll
    for (int k = 0; k < K; ++k) { q[k][0] = 0.0; q[k][1] = 0.0; }
    double n2 = 0.0;
    const float2* __restrict__ yrow = sY + lane * RS;
    // Coefficient registers of this group and of the next one.  The fetches go out for every class, active or
    // not, one group ahead of their use: a fetch under a branch would make every wait for a group's coefficients
    // a wait for all fetches in flight, the next group's included.  The two register sets swap roles from group
    // to group (the loop body handles two groups), so nothing is moved between them.
    double ca[K], cb[K];
#pragma unroll
    for (int k = 0; k < K; ++k) ca[k] = cf[k * CP];
    int ri = 0, j0 = 0;                      // wave-uniform: row and first column of the group
    double ar, ai;
    {
      const float2 a = yrow[0];
      ar = a.x;
      ai = a.y;
    }
    auto group = [&](const double (&ccur)[K], double (&cnxt)[K], int g) {
      const int gn = g + 1 < groups ? g + 1 : g;
#pragma unroll
      for (int k = 0; k < K; ++k) cnxt[k] = cf[k * CP + 16 * gn];
      const float2* __restrict__ yb = yrow + j0;
      const int cnt = __builtin_amdgcn_readfirstlane(D - j0);   // items of the group: 8, fewer at the end of a row
      // The group's items (ri, j0 + u), u < cnt, against the row-broadcast coefficients 2 u and 2 u + 1.  All 8
      // are formed, whatever cnt is: the reads beyond the row land in the rows of the following frames or, for
      // the last frame, in the weights behind the tile, and what is formed from them is not used.  (Forming the
      // upper four under a branch costs more than it saves: the compiler then clears their registers first.)
      double re[8], im[8];
      auto form = [&](int u) {
        const float2 bq = yb[u];
        const double br = bq.x, bi = bq.y;
        re[u] = ar * br + ai * bi;
        im[u] = ai * br - ar * bi;
      };
#pragma unroll
      for (int u = 0; u < 8; ++u) form(u);
      if (j0 == ri) n2 += re[0];               // the diagonal item: |y_i|^2
      static_for<0, K>([&](auto KI) {
        constexpr int k = decltype(KI)::value;
        if (class_on(mask, k)) fma_bcast_run(q[k][0], q[k][1], ccur[k], re, im, cnt);
      });
      j0 += 8;
      if (j0 >= D) {                           // next row
        ++ri;
        j0 = ri;
        if (ri < D) {
          const float2 a = yrow[ri];
          ar = a.x;
          ai = a.y;
        }
      }
    };
    {
      int g = 0;
      for (; g + 1 < groups; g += 2) {
        group(ca, cb, g);
        group(cb, ca, g + 1);
      }
      if (g < groups) group(ca, cb, g);
    }
    // posterior over the active classes: pi_k / det B_k * q_k^-D, mantissa / exponent form
    const double n2c = fmax(n2, GSS_EPS_NORM_SQ);
    const double qfloor = GSS_EPS_Q * n2c;
    double rq[K], mant[K];
    int ex[K];
    int emax = -(1 << 28);
    static_for<0, K>([&](auto KI) {
      constexpr int k = KI.value;
      rq[k] = 0.0;
      mant[k] = 0.0;
      ex[k] = -(1 << 28);
      if (class_on(mask, k)) {
        const bool a = (abits >> k) & 1u;
        rq[k] = rcp_f64(fmax(q[k][0] + q[k][1], qfloor));
        const double u = rq[k] * n2c;
        const double mu = __builtin_amdgcn_frexp_mant(u);
        const int eu = __builtin_amdgcn_frexp_exp(u);
        const double pw = ipow_rt(mu, D);            // >= 2^-32
        mant[k] = cm[k] * __builtin_amdgcn_frexp_mant(pw);
        ex[k] = a ? ce[k] + eu * D + __builtin_amdgcn_frexp_exp(pw) : -(1 << 28);
        emax = ex[k] > emax ? ex[k] : emax;
      }
    });
    double v[K], Z = 0.0;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      int de = ex[k] - emax;
      de = de < -1100 ? -1100 : de;
      v[k] = ((abits >> k) & 1u) ? ldexp(mant[k], de) : 0.0;
      Z += v[k];
    }
    const double rz = Z > 0.0 ? rcp_f64(Z) : 0.0;
    if (FINAL) {
      if (valid && !(n2 >= GSS_EPS_NORM_SQ)) atomicOr(status, GSS_STATUS_ZERO_FRAME);
      static_for<0, K>([&](auto KI) {
        constexpr int k = KI.value;
        if (class_on(mask, k)) {
          if (t < Tmax) gamma[(((long)s * K + k) * F + f) * Tmax + t] = (float)(v[k] * rz);
        }
      });
      wave_lds_sync();                       // the tile is overwritten by the next iteration
      continue;
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const double g = v[k] * rz;
      nacc[k] += g;
      sW[lane * WS + k] = g * rq[k];
    }
    wave_lds_sync();
    // ---- phase 2 ----
    accumulate_items<K, NR>(sY, sW, RS, WS, oi, oj, mask, acc);
    wave_lds_sync();
  }
  if (FINAL) return;

  double* __restrict__ red = reinterpret_cast<double*>(lds_raw);
  reduce_items<K, NR>(acc, red, part + (long)blockIdx.x * M * K * 2, M, lane, wave);
#pragma unroll
  for (int k = 0; k < K; ++k) {
    double nv = nacc[k];
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) nv += __shfl_xor(nv, off, kWave);
    nacc[k] = nv;
  }
  __syncthreads();
  if (lane == 0) {
#pragma unroll
    for (int k = 0; k < K; ++k) red[wave * K + k] = nacc[k];
  }
  __syncthreads();
  if (threadIdx.x < K) {
    double sum = 0.0;
    for (int w = 0; w < kLargeWaves; ++w) sum += red[w * K + threadIdx.x];
    npart[(long)blockIdx.x * K + threadIdx.x] = sum;
  }
}

// In-place Gauss-Jordan inversion of the D x D Hermitian positive-definite matrix in (sMr, sMi), thread
// (i, j) = (tid / D, tid % D), all threads of the workgroup call it.  Returns det as mant * 2^exp.
__device__ __forceinline__ void gauss_jordan_large(double (*sMr)[33], double (*sMi)[33], int D, int i, int j, bool on,
                                                   uint32_t* status, uint32_t flag, double& detm, int& dete) {
  detm = 1.0;
  dete = 0;
  for (int p = 0; p < D; ++p) {
    double piv = sMr[p][p];
    if (!(piv > 1e-300)) {
      piv = 1e-300;
      if (threadIdx.x == 0) atomicOr(status, flag);
    }
    detm *= piv;
    dete += __builtin_amdgcn_frexp_exp(detm);
    detm = __builtin_amdgcn_frexp_mant(detm);
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
}

// ----------------------------------------------------------------------------------------------
// Factor kernel, 9 <= D <= 32: one wavefront per (segment, frequency, class), a workgroup = the K classes of a
// (segment, frequency).  The D x D matrix sits in the registers of the wavefront: lane (a, b) = (lane / 8,
// lane % 8) holds the BS x BS block of rows a BS .. and columns b BS .. (BS = ceil(D / 8); rows and columns
// beyond D are those of the identity and stay so).  In-place Gauss-Jordan sweeps without pivoting (B is Hermitian
// positive definite after the loading; the product of the pivots is det B): the lanes that hold pivot row p and
// pivot column p publish them in the wavefront's LDS, every lane reads back the entries of its own columns and
// rows.  Nothing is shared between wavefronts, so there is no workgroup barrier.
// ----------------------------------------------------------------------------------------------
template <int BS>
__global__ __launch_bounds__(kWave * GSS_MAX_K) void em_factor_large(
    const double* __restrict__ part, const double* __restrict__ npart,
    double* __restrict__ coef, double* __restrict__ cmant, int32_t* __restrict__ cexp, uint32_t* __restrict__ status,
    int D, int K, ChunkMap cmap, int weight_mode) {
  constexpr int W = 8 * BS;                                // padded matrix size
  __shared__ double sPiv[GSS_MAX_K][4][W];                 // per wavefront: pivot row (re, im), pivot column (re, im)
  extern __shared__ __attribute__((aligned(16))) double sCoef[];   // per wavefront: the class's coef_pitch(D) coefficients
  const int lane = threadIdx.x & (kWave - 1);
  const int k = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const long sf = blockIdx.x;
  const int a = lane >> 3, b = lane & 7;
  const int M = num_items(D);
  int C;
  const long slot0 = chunk_base(cmap, sf, C);
  double* __restrict__ rowR = sPiv[k][0];
  double* __restrict__ rowI = sPiv[k][1];
  double* __restrict__ colR = sPiv[k][2];
  double* __restrict__ colI = sPiv[k][3];

  // class counts: lane l < K adds the chunks' counts of class l (in chunk order)
  double nl = 0.0;
  if (lane < K)
    for (int c = 0; c < C; ++c) nl += npart[(slot0 + c) * K + lane];
  const double Nk = __shfl(nl, k, kWave);
  double Ntot = 0.0;
  for (int kk = 0; kk < K; ++kk) Ntot += __shfl(nl, kk, kWave);

  // the lane's block of R_k = sum over the chunks (in chunk order) of the packed partial sums; entry (i, j) with
  // i > j is the conjugate of item (j, i)
  double mr[BS][BS], mi[BS][BS];
  int item[BS][BS];
#pragma unroll
  for (int r = 0; r < BS; ++r)
#pragma unroll
    for (int c = 0; c < BS; ++c) {
      const int i = a * BS + r, j = b * BS + c;
      const int lo = i < j ? i : j, hi = i < j ? j : i;
      item[r][c] = (hi < D) ? item_index(lo, hi, D) : 0;
      mr[r][c] = 0.0;
      mi[r][c] = 0.0;
    }
  for (int ch = 0; ch < C; ++ch) {
    const double* __restrict__ pc = part + ((slot0 + ch) * (long)M * K + k) * 2;
#pragma unroll
    for (int r = 0; r < BS; ++r)
#pragma unroll
      for (int c = 0; c < BS; ++c) {
        const double2 v = *reinterpret_cast<const double2*>(pc + (long)item[r][c] * K * 2);
        mr[r][c] += v.x;
        mi[r][c] += v.y;
      }
  }
  double trl = 0.0;
#pragma unroll
  for (int r = 0; r < BS; ++r)
#pragma unroll
    for (int c = 0; c < BS; ++c) {
      const int i = a * BS + r, j = b * BS + c;
      const bool in = i < D && j < D;
      mr[r][c] = in ? mr[r][c] : 0.0;
      mi[r][c] = in ? (i < j ? mi[r][c] : (i > j ? -mi[r][c] : 0.0)) : 0.0;
      if (r == c && a == b) trl += mr[r][c];
    }
  const double tr = wave_sum_f64(trl);
  // B = D R / max(N, eps); dead if its trace <= eps; else rescaled to trace D (= R * D / tr R); loading delta I
  const double trB = (double)D * tr / fmax(Nk, GSS_EPS_N);
  const bool dead = !(trB > GSS_EPS_N);
  const double sc = dead ? 0.0 : (double)D / tr;
#pragma unroll
  for (int r = 0; r < BS; ++r)
#pragma unroll
    for (int c = 0; c < BS; ++c) {
      const int i = a * BS + r, j = b * BS + c;
      const bool in = i < D && j < D;
      double vr = dead ? 0.0 : mr[r][c] * sc, vi = dead ? 0.0 : mi[r][c] * sc;
      if (i == j) {
        vr = dead ? 1.0 : vr;
        vi = 0.0;
        vr = in ? vr + GSS_DELTA : 1.0;                    // beyond D: the identity
      }
      mr[r][c] = vr;
      mi[r][c] = vi;
    }

  double detm = 1.0;
  int dete = 0;
  // (kept as a loop: unrolled, the 8 BS sweeps are straight-line code that every wavefront runs once, and the
  // kernel then waits for instruction fetches most of the time)
#pragma unroll 1
  for (int pg = 0; pg < 8; ++pg) {
    static_for<0, BS>([&](auto PP) {
      constexpr int pp = decltype(PP)::value;
      const int p = pg * BS + pp;
      if (p < D) {                                         // the same in every lane
        if (a == pg) {
#pragma unroll
          for (int c = 0; c < BS; ++c) { rowR[b * BS + c] = mr[pp][c]; rowI[b * BS + c] = mi[pp][c]; }
        }
        if (b == pg) {
#pragma unroll
          for (int r = 0; r < BS; ++r) { colR[a * BS + r] = mr[r][pp]; colI[a * BS + r] = mi[r][pp]; }
        }
        wave_lds_sync();
        double piv = rowR[p];
        double pr[BS], pim[BS], cr[BS], cim[BS];
#pragma unroll
        for (int c = 0; c < BS; ++c) { pr[c] = rowR[b * BS + c]; pim[c] = rowI[b * BS + c]; }
#pragma unroll
        for (int r = 0; r < BS; ++r) { cr[r] = colR[a * BS + r]; cim[r] = colI[a * BS + r]; }
        wave_lds_sync();                                   // read before the next sweep writes
        if (!(piv > 1e-300)) {
          piv = 1e-300;
          if (lane == 0) atomicOr(status, GSS_STATUS_NONPD_B);
        }
        detm *= piv;
        dete += __builtin_amdgcn_frexp_exp(detm);
        detm = __builtin_amdgcn_frexp_mant(detm);
        const double rp = rcp_f64(piv);
        // Every entry takes m - (column entry)(row entry) / pivot.  With pivot - 1 in place of the column entry
        // of the pivot row this gives (row entry) / pivot there, and with pivot + 1 in place of the row entry of
        // the pivot column it gives -(column entry) / pivot there; the pivot itself becomes 1 / pivot.
        const bool prow = a == pg, pcol = b == pg;
        cr[pp] = prow ? piv - 1.0 : cr[pp];
        cim[pp] = prow ? 0.0 : cim[pp];
        pr[pp] = pcol ? piv + 1.0 : pr[pp];
        pim[pp] = pcol ? 0.0 : pim[pp];
#pragma unroll
        for (int r = 0; r < BS; ++r)
#pragma unroll
          for (int c = 0; c < BS; ++c) {
            const double air = cr[r], aii = cim[r], apr = pr[c], api = pim[c];
            mr[r][c] -= (air * apr - aii * api) * rp;
            mi[r][c] -= (air * api + aii * apr) * rp;
          }
        if (prow && pcol) { mr[pp][pp] = rp; mi[pp][pp] = 0.0; }
      }
    });
  }

  // coefficients of <A, y y^H> over the items, A = the Hermitian part of the computed inverse: the diagonal
  // entry, and A_ij + conj(A_ji) for i < j (not 2 A_ij: rounding leaves the computed inverse slightly
  // non-Hermitian, and for an ill-conditioned B, whose inverse has entries of 1e6, one triangle mirrored puts a
  // relative error of up to 1e-4 into the quadratic forms of the class's own frames, the Hermitian part 1e-10).
  // The two triangles meet in the wavefront's LDS: the owners of the upper triangle write, then the owners of the
  // lower triangle add their conjugates, and the coefficients leave in the pass kernel's layout as one contiguous run.
  const int CP = coef_pitch(D);
  double* __restrict__ cf = coef + (sf * K + k) * (long)CP;
  double* __restrict__ sCo = sCoef + (long)k * CP;
  for (int x = lane; x < CP; x += kWave) sCo[x] = 0.0;     // the padding of the groups stays zero
  wave_lds_sync();
  int cpos[BS][BS];
#pragma unroll
  for (int r = 0; r < BS; ++r)
#pragma unroll
    for (int c = 0; c < BS; ++c) {
      const int i = a * BS + r, j = b * BS + c;
      const int lo = i < j ? i : j, hi = i < j ? j : i;
      cpos[r][c] = (hi < D) ? coef_pos(lo, hi, D) : 0;
    }
#pragma unroll
  for (int r = 0; r < BS; ++r)
#pragma unroll
    for (int c = 0; c < BS; ++c) {
      const int i = a * BS + r, j = b * BS + c;
      if (i <= j && j < D) *reinterpret_cast<double2*>(sCo + cpos[r][c]) = make_double2(mr[r][c], i == j ? 0.0 : mi[r][c]);
    }
  wave_lds_sync();
#pragma unroll
  for (int r = 0; r < BS; ++r)
#pragma unroll
    for (int c = 0; c < BS; ++c) {
      const int i = a * BS + r, j = b * BS + c;
      if (i > j && i < D) {                                // entry (i, j) of the lower triangle: item (j, i)
        double2 v = *reinterpret_cast<double2*>(sCo + cpos[r][c]);
        v.x += mr[r][c];
        v.y -= mi[r][c];
        *reinterpret_cast<double2*>(sCo + cpos[r][c]) = v;
      }
    }
  wave_lds_sync();
  for (int x = lane; x < CP; x += kWave) cf[x] = sCo[x];
  if (lane == 0) {
    const double pi = weight_mode == 1 ? Nk / fmax(Ntot, GSS_EPS_N) : 1.0 / (double)K;
    const double cst = fmax(pi, GSS_EPS_PI) / detm;
    cmant[sf * K + k] = __builtin_amdgcn_frexp_mant(cst);
    cexp[sf * K + k] = __builtin_amdgcn_frexp_exp(cst) - dete;
  }
}

// ----------------------------------------------------------------------------------------------
// MVDR, 9 <= D <= 32
// ----------------------------------------------------------------------------------------------
template <int NR>
__global__ __launch_bounds__(kWave * kLargeWaves) void mvdr_cov_large(
    gss_yview yv, const float* __restrict__ gamma, const int32_t* __restrict__ T_len,
    const int32_t* __restrict__ target, double* __restrict__ part, uint32_t* __restrict__ status,
    int F, int Tmax, int D, int K, ChunkMap cmap, int RS, int tile_bytes) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  constexpr int WS = 3;
  const int M = num_items(D);
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  long sf;
  int chunk, tiles_per_chunk;
  chunk_decode(cmap, blockIdx.x, sf, chunk, tiles_per_chunk);
  const int s = (int)(sf / F);
  const int f = (int)(sf % F);
  int T;
  const float2* __restrict__ Yrow = y_row(yv, T_len, s, f, D, Tmax, T);
  int tgt = target[s];
  if (tgt < 0 || tgt >= K) {
    if (threadIdx.x == 0 && chunk == 0 && f == 0) atomicOr(status, GSS_STATUS_BAD_TARGET);
    tgt = tgt < 0 ? 0 : K - 1;
  }
  float2* __restrict__ sY = reinterpret_cast<float2*>(lds_raw + (size_t)wave * tile_bytes);
  double* __restrict__ sW = reinterpret_cast<double*>(lds_raw + (size_t)wave * tile_bytes + (size_t)kWave * RS * sizeof(float2));
  const float* __restrict__ grow = gamma + ((long)s * K * F + f) * Tmax;
  const long gk = (long)F * Tmax;

  int oi[NR], oj[NR];
  double acc[NR][2][2];
#pragma unroll
  for (int n = 0; n < NR; ++n) {
    int m = lane + kWave * n;
    if (m >= M) m = 0;
    item_ij(m, D, oi[n], oj[n]);
    acc[n][0][0] = acc[n][0][1] = acc[n][1][0] = acc[n][1][1] = 0.0;
  }
  const int tile_lo = chunk * tiles_per_chunk;
  int tile_hi = tile_lo + tiles_per_chunk;
  const int tile_end = (T + kWave - 1) / kWave;
  tile_hi = tile_hi < tile_end ? tile_hi : tile_end;
  for (int tile = tile_lo + wave; tile < tile_hi; tile += kLargeWaves) {
    const int t0 = tile * kWave;
    const int t = t0 + lane;
    const bool valid = t < T;
    load_tile(Yrow, t0, T, D, RS, sY, lane);
    double wt = 0.0, wb = 0.0;
    for (int k = 0; k < K; ++k) {
      const double g = (double)grow[k * gk + (valid ? t : 0)];
      if (k == tgt) wt = g; else wb += g;
    }
    sW[lane * WS + 0] = valid ? wt : 0.0;
    sW[lane * WS + 1] = valid ? wb : 0.0;
    wave_lds_sync();
    accumulate_items<2, NR>(sY, sW, RS, WS, oi, oj, 3u, acc);
    wave_lds_sync();
  }
  double* __restrict__ red = reinterpret_cast<double*>(lds_raw);
  reduce_items<2, NR>(acc, red, part + (long)blockIdx.x * M * 4, M, lane, wave);
}

// One workgroup per (segment, frequency), D*D active threads.  H[sf][r][d], pw[sf][r][2] as for D <= 8.
__global__ __launch_bounds__(1024) void mvdr_solve_large(
    const double* __restrict__ part, double2* __restrict__ H, double* __restrict__ pw,
    uint32_t* __restrict__ status, int D, ChunkMap cmap) {
  __shared__ double sKr[32][33], sKi[32][33], sBr[32][33], sBi[32][33], sMr[32][33], sMi[32][33];
  double (*sGr)[33] = sMr;   // G and then H overwrite the inverse once it has been consumed
  double (*sGi)[33] = sMi;
  const int M = num_items(D);
  const long sf = blockIdx.x;
  int C;
  const long slot0 = chunk_base(cmap, sf, C);
  const int tid = threadIdx.x;
  const int i = tid / D, j = tid % D;
  const bool on = tid < D * D;
  if (on && i <= j) {
    const int m = item_index(i, j, D);
    double kr = 0.0, ki = 0.0, br = 0.0, bi = 0.0;
    for (int c = 0; c < C; ++c) {
      const double* p = part + ((slot0 + c) * (long)M + m) * 4;     // [k = 0 target, 1 background][re, im]
      kr += p[0]; ki += p[1]; br += p[2]; bi += p[3];
    }
    if (i == j) { ki = 0.0; bi = 0.0; }
    sKr[i][j] = kr; sKi[i][j] = ki; sBr[i][j] = br; sBi[i][j] = bi;
    if (i != j) { sKr[j][i] = kr; sKi[j][i] = -ki; sBr[j][i] = br; sBi[j][i] = -bi; }
  }
  __syncthreads();
  double trb = 0.0, trk = 0.0;
  for (int r = 0; r < D; ++r) { trb += sBr[r][r]; trk += sKr[r][r]; }
  if (!(trb > 0.0)) {
    if (trk > 0.0 && tid == 0) atomicOr(status, GSS_STATUS_NONPD_PHI);
    if (on) H[(sf * D + j) * D + i] = make_double2(0.0, 0.0);
    if (tid < D) { pw[(sf * D + tid) * 2 + 0] = 0.0; pw[(sf * D + tid) * 2 + 1] = 0.0; }
    return;
  }
  __syncthreads();
  if (on) {
    if (i == j) sBr[i][i] += GSS_DELTA_BF * trb / (double)D;
  }
  __syncthreads();
  if (on) { sMr[i][j] = sBr[i][j]; sMi[i][j] = sBi[i][j]; }
  __syncthreads();
  double detm;
  int dete;
  gauss_jordan_large(sMr, sMi, D, i, j, on, status, GSS_STATUS_NONPD_PHI, detm, dete);
  double gr = 0.0, gi = 0.0;
  if (on) {
    for (int m = 0; m < D; ++m) {
      const double ar = sMr[i][m], ai = sMi[i][m], br = sKr[m][j], bi = sKi[m][j];
      gr += ar * br - ai * bi;
      gi += ar * bi + ai * br;
    }
  }
  __syncthreads();
  if (on) { sGr[i][j] = gr; sGi[i][j] = gi; }
  __syncthreads();
  double tr = 0.0;
  for (int r = 0; r < D; ++r) tr += sGr[r][r];
  const double inv = 1.0 / (tr + GSS_EPS_TRACE);
  __syncthreads();
  if (on) {
    const double hr = sGr[i][j] * inv, hi = sGi[i][j] * inv;
    H[(sf * D + j) * D + i] = make_double2(hr, hi);
    sGr[i][j] = hr; sGi[i][j] = hi;
  }
  __syncthreads();
  if (tid < D) {
    const int r = tid;
    double pk = 0.0, pb = 0.0;
    for (int a = 0; a < D; ++a) {
      double tkr = 0.0, tki = 0.0, tbr = 0.0, tbi = 0.0;
      for (int b = 0; b < D; ++b) {
        const double hr = sGr[b][r], hi = sGi[b][r];
        tkr += sKr[a][b] * hr - sKi[a][b] * hi;  tki += sKr[a][b] * hi + sKi[a][b] * hr;
        tbr += sBr[a][b] * hr - sBi[a][b] * hi;  tbi += sBr[a][b] * hi + sBi[a][b] * hr;
      }
      const double hr = sGr[a][r], hi = sGi[a][r];
      pk += hr * tkr + hi * tki;
      pb += hr * tbr + hi * tbi;
    }
    pw[(sf * D + r) * 2 + 0] = pk;
    pw[(sf * D + r) * 2 + 1] = pb;
  }
}

__global__ __launch_bounds__(256) void mvdr_apply_large(
    gss_yview yv, const double2* __restrict__ H, const int32_t* __restrict__ ref,
    const int32_t* __restrict__ T_len, float2* __restrict__ X, int F, int Tmax, int D, int C, int frames_per_chunk,
    int ref_per_f) {
  __shared__ double2 sh[GSS_MAX_D];
  const int chunk = blockIdx.x % C;
  const long sf = blockIdx.x / C;
  const int s = (int)(sf / F);
  int T;
  const float2* __restrict__ Yrow = y_row(yv, T_len, s, (int)(sf % F), D, Tmax, T);
  int r = ref[ref_per_f ? sf : (long)s];
  r = r < 0 ? 0 : (r >= D ? D - 1 : r);
  if (threadIdx.x < D) sh[threadIdx.x] = H[(sf * D + r) * D + threadIdx.x];
  __syncthreads();
  float2* __restrict__ Xrow = X + sf * (long)Tmax;
  const int t_lo = chunk * frames_per_chunk;
  int t_hi = t_lo + frames_per_chunk;
  t_hi = t_hi < Tmax ? t_hi : Tmax;
  for (int t = t_lo + threadIdx.x; t < t_hi; t += blockDim.x) {
    double xr = 0.0, xi = 0.0;
    if (t < T) {
      for (int d = 0; d < D; ++d) {
        const float2 v = Yrow[(long)t * D + d];
        const double2 h = sh[d];
        xr += h.x * (double)v.x + h.y * (double)v.y;
        xi += h.x * (double)v.y - h.y * (double)v.x;
      }
    }
    Xrow[t] = make_float2((float)xr, (float)xi);
  }
}

struct LargePlan {
  int RS, tile_bytes, lds_bytes;
};

// LDS geometry of the tile kernels: per wavefront a tile of 64 frame rows of RS float2 plus the weights.
LargePlan plan_large(int D, int KW) {
  LargePlan p;
  p.RS = D + 1;                                            // float2 per frame row (odd: spreads the banks)
  const int ws = KW | 1;
  p.tile_bytes = (int)gss_align_up((size_t)kWave * p.RS * sizeof(float2) + (size_t)kWave * ws * sizeof(double), 16);
  const int red = num_items(D) * KW * 2 * (int)sizeof(double) + kLargeWaves * KW * (int)sizeof(double);
  const int tiles_b = kLargeWaves * p.tile_bytes;
  p.lds_bytes = tiles_b > red ? tiles_b : red;
  return p;
}

// Resident workgroup slots of a tile kernel with its dynamic LDS size.
template <typename Kern>
long large_slots(const gss_ctx* ctx, Kern kern, int lds_bytes) {
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kWave * kLargeWaves, (size_t)lds_bytes) != hipSuccess ||
      per_cu < 1)
    per_cu = 1;
  return (long)ctx->num_cu * per_cu;
}

template <int K, int NR>
int run_em_large(gss_ctx* ctx, const gss_yview& Y, const uint8_t* act, const int32_t* T_len, int S, int F, int Tmax,
                 int D, int iters, int weight_mode, float* gamma, hipStream_t st) {
  const long n_sf = (long)S * F;
  const int M = num_items(D);
  const LargePlan p = plan_large(D, K);
  if (hipFuncSetAttribute((const void*)em_pass_large<K, NR, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                          p.lds_bytes) != hipSuccess ||
      hipFuncSetAttribute((const void*)em_pass_large<K, NR, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                          p.lds_bytes) != hipSuccess)
    return GSS_EHIP;
  // the factor kernel stages every class's coefficients in LDS (up to 80 KB: 8 classes of 32 channels)
  const int factor_lds = K * coef_pitch(D) * (int)sizeof(double);
  const void* factor_kern = D <= 16 ? (const void*)em_factor_large<2> : D <= 24 ? (const void*)em_factor_large<3>
                                                                                 : (const void*)em_factor_large<4>;
  if (hipFuncSetAttribute(factor_kern, hipFuncAttributeMaxDynamicSharedMemorySize, factor_lds) != hipSuccess) return GSS_EHIP;
  const int tiles = (Tmax + kWave - 1) / kWave;
  const long slots = large_slots(ctx, em_pass_large<K, NR, false>, p.lds_bytes);
  const ChunkMap acc_map = plan_chunk_map(slots, n_sf, tiles, kLargeWaves, 0, true);
  const ChunkMap fin_map = plan_chunk_map(large_slots(ctx, em_pass_large<K, NR, true>, p.lds_bytes), n_sf, tiles,
                                          kLargeWaves, 0, true);
  const long wgs_acc = chunk_map_wgs(acc_map, n_sf), wgs_fin = chunk_map_wgs(fin_map, n_sf);
  if (wgs_acc > 0x7fffffffL || wgs_fin > 0x7fffffffL || n_sf * K > 0x7fffffffL) return GSS_EUNSUPPORTED;
  size_t o = 0;
  const size_t off_coef = o;  o = gss_align_up(o + (size_t)n_sf * K * coef_pitch(D) * sizeof(double), 256);
  const size_t off_cm = o;    o = gss_align_up(o + (size_t)n_sf * K * sizeof(double), 256);
  const size_t off_ce = o;    o = gss_align_up(o + (size_t)n_sf * K * sizeof(int32_t), 256);
  const size_t off_part = o;  o = gss_align_up(o + (size_t)wgs_acc * M * K * 2 * sizeof(double), 256);
  const size_t off_npart = o; o = gss_align_up(o + (size_t)wgs_acc * K * sizeof(double), 256);
  const size_t off_abyte = o; o = gss_align_up(o + (size_t)S * Tmax, 256);
  const size_t off_tmask = o; o = gss_align_up(o + (size_t)S * tiles * sizeof(uint32_t), 256);
  if ((long)S * tiles > 0x7fffffffL) return GSS_EUNSUPPORTED;
  int rc = gss_ensure_scratch(ctx, o);
  if (rc != GSS_OK) return rc;
  char* base = (char*)ctx->scratch;
  uint8_t* abyte = (uint8_t*)(base + off_abyte);
  uint32_t* tmask = (uint32_t*)(base + off_tmask);
  double* coef = (double*)(base + off_coef);
  double* cm = (double*)(base + off_cm);
  int32_t* ce = (int32_t*)(base + off_ce);
  double* part = (double*)(base + off_part);
  double* npart = (double*)(base + off_npart);
  const dim3 block(kWave * kLargeWaves);
  hipLaunchKernelGGL(em_init_coef_large, dim3(1024), dim3(256), 0, st, coef, cm, ce, D, K, n_sf);
  hipLaunchKernelGGL(em_pack_activity, dim3((unsigned)(S * tiles)), dim3(kWave), 0, st, Y, act, T_len, abyte, tmask, K,
                     Tmax, tiles);
  for (int it = 0; it < iters; ++it) {
    gss_profile_begin(ctx, 0, st);
    hipLaunchKernelGGL((em_pass_large<K, NR, false>), dim3((unsigned)wgs_acc), block, p.lds_bytes, st, Y, abyte, tmask, T_len,
                       coef, cm, ce, part, npart, (float*)nullptr, ctx->status, F, Tmax, D, acc_map, p.RS, p.tile_bytes);
    gss_profile_end(ctx, 0, st);
    gss_profile_begin(ctx, 1, st);
    if (D <= 16)
      hipLaunchKernelGGL(em_factor_large<2>, dim3((unsigned)n_sf), dim3(kWave * K), factor_lds, st, part, npart, coef, cm, ce,
                         ctx->status, D, K, acc_map, weight_mode);
    else if (D <= 24)
      hipLaunchKernelGGL(em_factor_large<3>, dim3((unsigned)n_sf), dim3(kWave * K), factor_lds, st, part, npart, coef, cm, ce,
                         ctx->status, D, K, acc_map, weight_mode);
    else
      hipLaunchKernelGGL(em_factor_large<4>, dim3((unsigned)n_sf), dim3(kWave * K), factor_lds, st, part, npart, coef, cm, ce,
                         ctx->status, D, K, acc_map, weight_mode);
    gss_profile_end(ctx, 1, st);
  }
  hipLaunchKernelGGL((em_pass_large<K, NR, true>), dim3((unsigned)wgs_fin), block, p.lds_bytes, st, Y, abyte, tmask, T_len, coef,
                     cm, ce, (double*)nullptr, (double*)nullptr, gamma, ctx->status, F, Tmax, D, fin_map, p.RS, p.tile_bytes);
  if (hipGetLastError() != hipSuccess) return GSS_EHIP;
  return GSS_OK;
}

template <int K>
int dispatch_nr(gss_ctx* ctx, const gss_yview& Y, const uint8_t* act, const int32_t* T_len, int S, int F, int Tmax,
                int D, int iters, int weight_mode, float* gamma, hipStream_t st) {
  const int nr = (num_items(D) + kWave - 1) / kWave;       // 1 .. 9
  if (nr <= 3) return run_em_large<K, 3>(ctx, Y, act, T_len, S, F, Tmax, D, iters, weight_mode, gamma, st);
  if (nr <= 5) return run_em_large<K, 5>(ctx, Y, act, T_len, S, F, Tmax, D, iters, weight_mode, gamma, st);
  if (nr <= 7) return run_em_large<K, 7>(ctx, Y, act, T_len, S, F, Tmax, D, iters, weight_mode, gamma, st);
  return run_em_large<K, 9>(ctx, Y, act, T_len, S, F, Tmax, D, iters, weight_mode, gamma, st);
}

template <int NR>
int run_mvdr_large(gss_ctx* ctx, const gss_yview& Y, const float* gamma, const int32_t* T_len, int S, int F, int Tmax,
                   int D, int K, const int32_t* target, int32_t* ref, int ref_per_f, float2* X, hipStream_t st) {
  const long n_sf = (long)S * F;
  const int M = num_items(D);
  const LargePlan p = plan_large(D, 2);
  if (hipFuncSetAttribute((const void*)mvdr_cov_large<NR>, hipFuncAttributeMaxDynamicSharedMemorySize, p.lds_bytes) !=
      hipSuccess)
    return GSS_EHIP;
  const int tiles = (Tmax + kWave - 1) / kWave;
  const ChunkMap cmap = plan_chunk_map(large_slots(ctx, mvdr_cov_large<NR>, p.lds_bytes), n_sf, tiles, kLargeWaves, 0, true);
  const long wgs = chunk_map_wgs(cmap, n_sf);
  if (wgs > 0x7fffffffL) return GSS_EUNSUPPORTED;
  size_t o = 0;
  const size_t off_part = o; o = gss_align_up(o + (size_t)wgs * M * 4 * sizeof(double), 256);
  const size_t off_H = o;    o = gss_align_up(o + (size_t)n_sf * D * D * sizeof(double2), 256);
  const size_t off_pw = o;   o = gss_align_up(o + (size_t)n_sf * D * 2 * sizeof(double), 256);
  int rc = gss_ensure_scratch(ctx, o);
  if (rc != GSS_OK) return rc;
  char* base = (char*)ctx->scratch;
  double* part = (double*)(base + off_part);
  double2* H = (double2*)(base + off_H);
  double* pw = (double*)(base + off_pw);
  hipLaunchKernelGGL((mvdr_cov_large<NR>), dim3((unsigned)wgs), dim3(kWave * kLargeWaves), p.lds_bytes, st, Y, gamma, T_len,
                     target, part, ctx->status, F, Tmax, D, K, cmap, p.RS, p.tile_bytes);
  const int sthreads = (D * D + 63) / 64 * 64;
  hipLaunchKernelGGL(mvdr_solve_large, dim3((unsigned)n_sf), dim3(sthreads), 0, st, part, H, pw, ctx->status, D, cmap);
  gss_launch_mvdr_ref(pw, ref, ctx->status, S, F, D, ref_per_f, st);
  const int fpc = 1024;
  const int CA = (Tmax + fpc - 1) / fpc;
  if (n_sf * CA > 0x7fffffffL) return GSS_EUNSUPPORTED;
  hipLaunchKernelGGL(mvdr_apply_large, dim3((unsigned)(n_sf * CA)), dim3(256), 0, st, Y, H, ref, T_len, X, F, Tmax, D,
                     CA, fpc, ref_per_f);
  if (hipGetLastError() != hipSuccess) return GSS_EHIP;
  return GSS_OK;
}

}  // namespace
