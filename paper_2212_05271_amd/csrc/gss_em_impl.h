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
#pragma once

#include "gss_internal.h"

#include "gss_device.h"

namespace {

// ----------------------------------------------------------------------------------------------
// Coefficient initialisation: B = I, log-term 0  (pass 0).
// coef[sf][k][E] packed as gss_packed_row(); the class constant pi_k / det B_k is kept as
// cmant * 2^cexp with cmant in [0.5, 1).
// ----------------------------------------------------------------------------------------------
__global__ void em_init_coef(double* __restrict__ coef, double* __restrict__ cmant, int32_t* __restrict__ cexp,
                             int D, int K, long n_sf) {
  const int E = D * D;
  long total = n_sf * (long)K * E;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    int e = (int)(i % E);
    // diagonal entries sit at gss_packed_row(r, D)
    double v = 0.0;
    for (int r = 0; r < D; ++r)
      if (e == gss_packed_row(r, D)) v = 1.0;
    coef[i] = v;
  }
  long nl = n_sf * (long)K;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nl; i += (long)gridDim.x * blockDim.x) {
    cmant[i] = 0.5;
    cexp[i] = 1;
  }
}

// ----------------------------------------------------------------------------------------------
// Pass kernel for D <= 8.  Workgroup = kPassWaves wavefronts that all work on the same
// (segment, frequency), so that the class coefficients they stream through the scalar cache are shared;
// every wavefront owns whole tiles of 64 frames and a private LDS region, and there is no workgroup
// barrier inside the tile loop.
//
// Phase 1 (lane = frame): q_k = <coef_k, y y^H> with the outer product generated entry by entry in fp64
//   and the coefficients wave-uniform (scalar loads); posterior over the active classes as
//   pi_k / det B_k * q_k^-D in (mantissa, exponent) form, fp64, no log/exp; weights w_k = gamma_k / q_k.
//   y (as fp64) and w go to the wavefront's LDS tile.
// Phase 2 (lane = (frame group tg, channel eg), 8 x 8; frames tg, tg+8, ... of the tile): lane type eg = i
//   owns the entries y_i conj(y_b) for b = i+1, i+2, i+3 (mod 8), and either the pair (i, i+4) (i < 4) or
//   the real diagonal entries of channels i and i-4 (i >= 4): 8 real entries per lane, all 64 of the packed
//   Hermitian 8 x 8 matrix over the 8 lane types, the same instructions for every lane except the last two
//   entries.  For its 8 frames per tile a lane reads 5 channels of y and the K weights, forms its 8
//   entries exactly and accumulates R_k[e] += w_k * P[e] in fp64.  Channels >= D are zero padding.
//   The accumulators stay in registers across the tiles of the chunk.
//
// Grid: blockIdx.x = chunk + C * (f + F * s).  A chunk is `tiles_per_chunk` tiles of 64 frames, dealt to
// the wavefronts round-robin.
// ----------------------------------------------------------------------------------------------


// Entries of the packed outer product per group of scalar coefficient loads (2 or 4 doubles per class);
// two groups are in SGPRs at a time, 2 * K * G * 2 registers of the 100 or so there are.
__host__ __device__ constexpr int coef_group(int K) { return K <= 5 ? 4 : 2; }

// Frames per lane in phase 1.  Every class coefficient that comes through the scalar path is applied to
// kNF frames; the scalar data path returns about one dword per clock per pair of compute units, so
// at kNF = 1 it is as busy as the vector ALUs.
constexpr int kNF = 2;

// One unit of work of a wavefront: NF consecutive tiles of 64 frames starting at frame t0.
template <int D, int K, int NF, bool FINAL>
__device__ __forceinline__ void pass_unit(
    const float2* __restrict__ Yrow, const uint8_t* __restrict__ arow, const double* __restrict__ cf,
    const double* __restrict__ cm, const int32_t* __restrict__ ce, float* __restrict__ gamma_row /* + k*F*Tmax */,
    uint32_t* __restrict__ status, long gamma_kstride, int T, int Tmax, int t0, int lane, double* __restrict__ sY,
    double* __restrict__ sW,
    double (&acc)[8][K], double (&nacc)[K]) {
  constexpr int E = D * D;
  constexpr int WS = K | 1;
  const int tg = lane >> 3, eg = lane & 7;

  // ---- phase 1: load y ----
  // A lane whose frame lies beyond T reads frame 0 instead (it exists whenever a tile is processed at all, or is
  // padding in the final pass); its activity bits are forced to zero, so its posterior and weights are zero.
  int t[NF];
  bool valid[NF];
  double yr[NF][D], yi[NF][D];
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    t[f] = t0 + f * kWave + lane;
    valid[f] = t[f] < T;
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const float2 v = Yrow[(long)(valid[f] ? t[f] : 0) * D + d];
      yr[f][d] = (double)v.x;
      yi[f][d] = (double)v.y;
    }
  }
  // activity bits of the lane's frames, fetched here so that the loads overlap the q loop
  unsigned abits[NF];
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    unsigned b = 0;
#pragma unroll
    for (int k = 0; k < K; ++k) b |= (arow[(long)k * Tmax + (valid[f] ? t[f] : 0)] != 0 ? 1u : 0u) << k;
    abits[f] = valid[f] ? b : 0u;
    asm volatile("" : "+v"(abits[f]));
  }

  // ---- q_k = <coef_k, y y^H> ----
  // The coefficients are wave-uniform and come through the scalar path straight into the FMAs as SGPR
  // operands, one group of G packed entries (K*G doubles) at a time, two groups in registers: the loads of
  // group g + 1 are issued during the arithmetic of group g.  Left alone, the compiler either hoists all
  // K*E loads out of the tile loop and spills them, or puts every load directly in front of its first use.
  // The empty asm statements steer it: the offset of group g + 1 comes into existence only after the first
  // product of group g (which is where the wait for group g's loads lands, with nothing else outstanding:
  // scalar loads may return out of order, so that wait is always for all of them), and every partial sum
  // passes through a fence at the end of its group, which keeps the group's arithmetic in place.
  double q[NF][K];
  double n2[NF];
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    n2[f] = 0.0;
#pragma unroll
    for (int k = 0; k < K; ++k) q[f][k] = 0.0;
  }
  constexpr int G = coef_group(K);
  constexpr int NG = (E + G - 1) / G;
  typedef const __attribute__((address_space(4))) double* const_ptr_t;
  const const_ptr_t cf4 = (const_ptr_t)(uintptr_t)cf;
  double ccur[K][G], cnxt[K][G];
  {
    int off0 = 0;
    asm volatile("" : "+s"(off0));            // opaque (uniform) offset: keeps the loads inside this unit
    const const_ptr_t c0 = cf4 + off0;
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
      for (int e = 0; e < G; ++e) ccur[k][e] = (e < E) ? c0[k * E + e] : 0.0;
  }
  static_for<0, NG>([&](auto GI) {
    constexpr int g = GI.value * G;
    constexpr int ng = (E - g) < G ? (E - g) : G;
    double Pg[NF][ng];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      static_for<0, ng>([&](auto EI) {
        constexpr int e = EI.value;
        Pg[f][e] = packed_entry<D, g + e>(yr[f], yi[f]);
        if constexpr (packed_part(g + e, D) == 0) n2[f] += Pg[f][e];
      });
    }
    q[0][0] = fma(ccur[0][0], Pg[0][0], q[0][0]);      // first use of this group: waits for its loads
    if constexpr (g + G < E) {
      int noff = g + G;
      asm volatile("" : "+s"(noff), "+v"(q[0][0]));   // the next group's offset exists only from here on
      const const_ptr_t cn = cf4 + noff;
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int e = 0; e < G; ++e) cnxt[k][e] = (g + G + e < E) ? cn[k * E + e] : 0.0;
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
#pragma unroll
      for (int e = 0; e < ng; ++e) {
#pragma unroll
        for (int f = 0; f < NF; ++f)
          if (!(k == 0 && e == 0 && f == 0)) q[f][k] = fma(ccur[k][e], Pg[f][e], q[f][k]);
      }
    }
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
      for (int k = 0; k < K; ++k) asm volatile("" : "+v"(q[f][k]));
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
      for (int e = 0; e < G; ++e) ccur[k][e] = cnxt[k][e];
  });

#pragma unroll
  for (int f = 0; f < NF; ++f) {
    // posterior over the active classes: pi_k / det B_k * q_k^-D with q_k = max(qraw_k / n2c, eps_q)
    const double n2c = fmax(n2[f], GSS_EPS_NORM_SQ);
    const double qfloor = GSS_EPS_Q * n2c;
    double rq[K], mant[K];
    int ex[K];
    bool a[K];
    int emax = -(1 << 28);
#pragma unroll
    for (int k = 0; k < K; ++k) {
      a[k] = (abits[f] >> k) & 1u;
      rq[k] = rcp_f64_fast(fmax(q[f][k], qfloor));        // 1 / (q_k * n2c): the M-step weight is gamma_k * rq
      const double u = rq[k] * n2c;                  // 1 / q_k
      const double mu = __builtin_amdgcn_frexp_mant(u);
      const int eu = __builtin_amdgcn_frexp_exp(u);
      const double pw = ipow<D>(mu);                 // in [2^-D, 1)
      mant[k] = cm[k] * __builtin_amdgcn_frexp_mant(pw);
      ex[k] = a[k] ? ce[k] + eu * D + __builtin_amdgcn_frexp_exp(pw) : -(1 << 28);
      emax = ex[k] > emax ? ex[k] : emax;
    }
    double v[K], Z = 0.0;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      int de = ex[k] - emax;
      de = de < -1100 ? -1100 : de;
      v[k] = a[k] ? ldexp(mant[k], de) : 0.0;
      Z += v[k];
    }
    const double rz = Z > 0.0 ? rcp_f64_fast(Z) : 0.0;
    if constexpr (FINAL) {
      if (valid[f] && !(n2[f] >= GSS_EPS_NORM_SQ)) atomicOr(status, GSS_STATUS_ZERO_FRAME);
      if (t[f] < Tmax) {
#pragma unroll
        for (int k = 0; k < K; ++k) gamma_row[k * gamma_kstride + t[f]] = (float)(v[k] * rz);
      }
    } else {
      // this tile's y and weights go to LDS, then phase 2 runs over it
      if (t0 + f * kWave >= T) break;              // uniform: nothing valid in this tile
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        double2 yv = make_double2(0.0, 0.0);
        if (d < D) yv = make_double2(yr[f][d < D ? d : 0], yi[f][d < D ? d : 0]);
        *reinterpret_cast<double2*>(&sY[lane * kYStride + 2 * d]) = yv;
      }
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const double g = v[k] * rz;
        nacc[k] += g;
        sW[lane * WS + k] = g * rq[k];
      }
      wave_lds_sync();

      // ---- phase 2 ----
      accumulate_tile<K, K | 1>(sY, sW, tg, eg, acc);
      wave_lds_sync();
    }
  }
}

template <int D, int K, bool FINAL>
__global__ __launch_bounds__(kWave * kPassWaves, 2) void em_pass_small(
    const float2* __restrict__ Y, const uint8_t* __restrict__ act, const int32_t* __restrict__ T_len,
    const double* __restrict__ coef, const double* __restrict__ cmant, const int32_t* __restrict__ cexp,
    double* __restrict__ part, double* __restrict__ npart, float* __restrict__ gamma, uint32_t* __restrict__ status,
    int F, int Tmax, ChunkMap cmap) {
  constexpr int E = D * D;
  constexpr int WS = K | 1;
  constexpr int kTileDoubles = kWave * kYStride + kWave * WS;
  // per-wavefront tiles; reused at the end for the cross-wavefront reduction (needs kPassWaves*(64*K+K))
  constexpr int kRedDoubles = kPassWaves * (64 * K + K);
  constexpr int kLdsDoubles = FINAL ? 1 : (kPassWaves * kTileDoubles > kRedDoubles ? kPassWaves * kTileDoubles : kRedDoubles);
  __shared__ __attribute__((aligned(16))) double lds[kLdsDoubles];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  long sf;
  int chunk, tiles_per_chunk;
  chunk_decode(cmap, blockIdx.x, sf, chunk, tiles_per_chunk);
  const int s = (int)((unsigned)sf / (unsigned)F);
  const int f = (int)((unsigned)sf % (unsigned)F);
  int T = T_len ? T_len[s] : Tmax;
  T = T < 0 ? 0 : (T > Tmax ? Tmax : T);
  const int t_end = FINAL ? Tmax : T;       // the final pass also writes the zero padding

  const double* __restrict__ cf = coef + sf * (long)(K * E);
  const double* __restrict__ cm = cmant + sf * K;
  const int32_t* __restrict__ ce = cexp + sf * K;
  double* __restrict__ sY = lds + (FINAL ? 0 : wave * kTileDoubles);
  double* __restrict__ sW = sY + (FINAL ? 0 : kWave * kYStride);

  double acc[8][K];
  double nacc[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    nacc[k] = 0.0;
#pragma unroll
    for (int n = 0; n < 8; ++n) acc[n][k] = 0.0;
  }
  const float2* __restrict__ Yrow = Y + sf * (long)Tmax * D;
  const uint8_t* __restrict__ arow = act + (long)s * K * Tmax;
  float* __restrict__ gamma_row = FINAL ? gamma + ((long)s * K * F + f) * Tmax : nullptr;
  const long gamma_kstride = (long)F * Tmax;

  // The chunk's tiles, as units of kNF tiles followed by single tiles, dealt to the wavefronts round-robin.
  const int tile_lo = chunk * tiles_per_chunk;
  int tile_hi = tile_lo + tiles_per_chunk;
  const int tile_end = (t_end + kWave - 1) / kWave;
  tile_hi = tile_hi < tile_end ? tile_hi : tile_end;
  const int n_tiles = tile_hi > tile_lo ? tile_hi - tile_lo : 0;
  // a chunk with no more tiles than wavefronts is dealt out tile by tile
  const int n_big = n_tiles <= kPassWaves ? 0 : n_tiles / kNF;
  const int n_units = n_big + (n_tiles - n_big * kNF);
  for (int u = wave; u < n_units; u += kPassWaves) {
    if (u < n_big) {
      pass_unit<D, K, kNF, FINAL>(Yrow, arow, cf, cm, ce, gamma_row, status, gamma_kstride, T, Tmax,
                                  (tile_lo + u * kNF) * kWave, lane, sY, sW, acc, nacc);
    } else {
      pass_unit<D, K, 1, FINAL>(Yrow, arow, cf, cm, ce, gamma_row, status, gamma_kstride, T, Tmax,
                                (tile_lo + n_big * kNF + (u - n_big)) * kWave, lane, sY, sW, acc, nacc);
    }
  }
  if (FINAL) return;

  // Reduce over the 8 frame groups and over the wavefronts; write the chunk's packed partial sums and counts.
  reduce_and_store_partials<D, K, true>(acc, nacc, sY, lds, part + (long)blockIdx.x * (K * E),
                                        npart + (long)blockIdx.x * K, lane, wave);
}

// ----------------------------------------------------------------------------------------------
// Factor kernel for D <= 8: one workgroup per (segment, frequency), one wavefront per class.
// Sums the chunk partials in a fixed order (deterministic), forms B = D R / N, regularises (trace D,
// + delta I; identity for a class without data), inverts by in-place Gauss-Jordan sweeps in fp64
// (pivots = Schur complements, positive for a Hermitian positive-definite matrix; their product is
// det B) and writes the packed coefficients of B^-1 and the class constant pi_k / det B_k of the next pass.
// ----------------------------------------------------------------------------------------------
template <int D, int K>
__global__ __launch_bounds__(kWave * K) void em_factor_small(
    const double* __restrict__ part, const double* __restrict__ npart,
    double* __restrict__ coef, double* __restrict__ cmant, int32_t* __restrict__ cexp, uint32_t* __restrict__ status,
    ChunkMap cmap, int weight_mode) {
  constexpr int E = D * D;
  __shared__ double sR[K][E];
  __shared__ double sMr[K][D][D], sMi[K][D][D];
  __shared__ double sN[K];

  const long sf = blockIdx.x;
  const int k = threadIdx.x / kWave;
  const int l = threadIdx.x % kWave;
  int C;
  const long slot0 = chunk_base(cmap, sf, C);

  if (l < E) {
    double r = 0.0;
    for (int c = 0; c < C; ++c) r += part[((slot0 + c) * K + k) * (long)E + l];
    sR[k][l] = r;
  }
  if (l == 0) {
    double n = 0.0;
    for (int c = 0; c < C; ++c) n += npart[(slot0 + c) * K + k];
    sN[k] = n;
  }
  __syncthreads();

  const int i = l / D, j = l % D;
  const bool on = l < E;
  double tr = 0.0;
#pragma unroll
  for (int r = 0; r < D; ++r) tr += sR[k][gss_packed_row(r, D)];
  const double Nk = sN[k];
  // B = D R / max(N, eps); dead if its trace <= eps; else rescale to trace D  (=> R * D / tr R)
  const double trB = (double)D * tr / fmax(Nk, GSS_EPS_N);
  const bool dead = !(trB > GSS_EPS_N);
  double mr = 0.0, mi = 0.0;
  if (on) {
    if (dead) {
      mr = (i == j) ? 1.0 : 0.0;
    } else {
      const double sc = (double)D / tr;
      if (i == j) {
        mr = sR[k][gss_packed_row(i, D)] * sc;
      } else {
        const int lo = i < j ? i : j, hi = i < j ? j : i;
        const int p = gss_packed_row(lo, D) + 1 + 2 * (hi - lo - 1);
        mr = sR[k][p] * sc;
        mi = sR[k][p + 1] * sc;
        if (i > j) mi = -mi;                 // lower triangle = conjugate
      }
    }
    if (i == j) mr += GSS_DELTA;
    sMr[k][i][j] = mr;
    sMi[k][i][j] = mi;
  }
  wave_lds_sync();          // from here on every wavefront works on its own class matrix only

  double detm = 1.0;   // det B = detm * 2^dete, renormalised after every pivot
  int dete = 0;
  for (int p = 0; p < D; ++p) {
    double piv = sMr[k][p][p];
    if (!(piv > 1e-300)) {
      piv = 1e-300;
      if (l == 0) atomicOr(status, GSS_STATUS_NONPD_B);
    }
    detm *= piv;
    dete += __builtin_amdgcn_frexp_exp(detm);
    detm = __builtin_amdgcn_frexp_mant(detm);
    const double rp = rcp_f64(piv);
    double nr = 0.0, ni = 0.0;
    if (on) {
      const double air = sMr[k][i][p], aii = sMi[k][i][p];
      const double apr = sMr[k][p][j], api = sMi[k][p][j];
      if (i == p && j == p) {
        nr = rp;
      } else if (i == p) {
        nr = apr * rp; ni = api * rp;
      } else if (j == p) {
        nr = -air * rp; ni = -aii * rp;
      } else {
        nr = sMr[k][i][j] - (air * apr - aii * api) * rp;
        ni = sMi[k][i][j] - (air * api + aii * apr) * rp;
      }
    }
    wave_lds_sync();
    if (on) { sMr[k][i][j] = nr; sMi[k][i][j] = ni; }
    wave_lds_sync();
  }

  // packed coefficients of q = sum_i A_ii P_ii + 2 sum_{i<j} (Re A_ij Re P_ij + Im A_ij Im P_ij), A = B^-1
  if (on && i <= j) {
    double* __restrict__ cf = coef + (sf * K + k) * (long)E;
    if (i == j) {
      cf[gss_packed_row(i, D)] = sMr[k][i][i];
    } else {
      const int p = gss_packed_row(i, D) + 1 + 2 * (j - i - 1);
      cf[p] = 2.0 * sMr[k][i][j];
      cf[p + 1] = 2.0 * sMi[k][i][j];
    }
  }
  if (l == 0) {
    double pi;
    if (weight_mode == 1) {
      double tot = 0.0;
      for (int kk = 0; kk < K; ++kk) tot += sN[kk];
      pi = Nk / fmax(tot, GSS_EPS_N);
    } else {
      pi = 1.0 / (double)K;
    }
    const double c = fmax(pi, GSS_EPS_PI) / detm;            // pi_k / det B_k = c * 2^-dete
    cmant[sf * K + k] = __builtin_amdgcn_frexp_mant(c);
    cexp[sf * K + k] = __builtin_amdgcn_frexp_exp(c) - dete;
  }
}

// ----------------------------------------------------------------------------------------------
// Host-side plan and dispatch
// ----------------------------------------------------------------------------------------------
struct EmPlan {
  ChunkMap acc;          // chunking of the accumulating passes
  ChunkMap fin;          // chunking of the final pass
  long wgs_acc, wgs_fin;
  size_t off_coef, off_cm, off_ce, off_part, off_npart, total;
};

EmPlan make_plan(const gss_ctx* ctx, long n_sf, int Tmax, int D, int K, int wgs_per_cu, int wgs_per_cu_fin) {
  EmPlan p;
  const int tiles = (Tmax + kWave - 1) / kWave;
  const int round_up = kPassWaves * kNF;               // a chunk is a whole number of rounds of units
  const long slots = (long)ctx->num_cu * wgs_per_cu;
  p.acc = plan_chunk_map(slots, n_sf, tiles, round_up, 0, true);
  p.wgs_acc = chunk_map_wgs(p.acc, n_sf);
  p.fin = plan_chunk_map((long)ctx->num_cu * wgs_per_cu_fin, n_sf, tiles, round_up, 0, true);
  p.wgs_fin = chunk_map_wgs(p.fin, n_sf);
  const size_t E = (size_t)D * D;
  size_t o = 0;
  p.off_coef = o;  o = gss_align_up(o + (size_t)n_sf * K * E * sizeof(double) + 64, 256);
  p.off_cm = o;    o = gss_align_up(o + (size_t)n_sf * K * sizeof(double), 256);
  p.off_ce = o;    o = gss_align_up(o + (size_t)n_sf * K * sizeof(int32_t), 256);
  p.off_part = o;  o = gss_align_up(o + (size_t)p.wgs_acc * K * E * sizeof(double), 256);
  p.off_npart = o; o = gss_align_up(o + (size_t)p.wgs_acc * K * sizeof(double), 256);
  p.total = o;
  return p;
}

template <int D, int K>
int run_small(gss_ctx* ctx, const float2* Y, const uint8_t* act, const int32_t* T_len, int S, int F, int Tmax,
              int iters, int weight_mode, float* gamma, hipStream_t st) {
  const long n_sf = (long)S * F;
  // resident workgroups per compute unit of the two pass kernels: asked once per instantiation
  static const int wgs_per_cu = resident_wgs(em_pass_small<D, K, false>, kWave * kPassWaves, 2);
  static const int wgs_per_cu_fin = resident_wgs(em_pass_small<D, K, true>, kWave * kPassWaves, 2);
  const EmPlan p = make_plan(ctx, n_sf, Tmax, D, K, wgs_per_cu, wgs_per_cu_fin);
  int rc = gss_ensure_scratch(ctx, p.total);
  if (rc != GSS_OK) return rc;
  char* base = (char*)ctx->scratch;
  double* coef = (double*)(base + p.off_coef);
  double* cm = (double*)(base + p.off_cm);
  int32_t* ce = (int32_t*)(base + p.off_ce);
  double* part = (double*)(base + p.off_part);
  double* npart = (double*)(base + p.off_npart);

  if (p.wgs_acc > 0x7fffffffL || p.wgs_fin > 0x7fffffffL) return GSS_EUNSUPPORTED;
  const dim3 block(kWave * kPassWaves);
  hipLaunchKernelGGL(em_init_coef, dim3(1024), dim3(256), 0, st, coef, cm, ce, D, K, n_sf);
  for (int it = 0; it < iters; ++it) {
    gss_profile_begin(ctx, 0, st);
    hipLaunchKernelGGL((em_pass_small<D, K, false>), dim3((unsigned)p.wgs_acc), block, 0, st, Y, act, T_len, coef, cm, ce,
                       part, npart, (float*)nullptr, ctx->status, F, Tmax, p.acc);
    gss_profile_end(ctx, 0, st);
    gss_profile_begin(ctx, 1, st);
    hipLaunchKernelGGL((em_factor_small<D, K>), dim3((unsigned)n_sf), dim3(kWave * K), 0, st, part, npart, coef, cm, ce,
                       ctx->status, p.acc, weight_mode);
    gss_profile_end(ctx, 1, st);
  }
  hipLaunchKernelGGL((em_pass_small<D, K, true>), dim3((unsigned)p.wgs_fin), block, 0, st, Y, act, T_len, coef, cm, ce,
                     (double*)nullptr, (double*)nullptr, gamma, ctx->status, F, Tmax, p.fin);
  if (hipGetLastError() != hipSuccess) return GSS_EHIP;
  return GSS_OK;
}

template <int D>
int dispatch_k(gss_ctx* ctx, const float2* Y, const uint8_t* act, const int32_t* T_len, int S, int F, int Tmax,
               int K, int iters, int weight_mode, float* gamma, hipStream_t st) {
  switch (K) {
#define GSS_CASE_K(KK) \
  case KK: return run_small<D, KK>(ctx, Y, act, T_len, S, F, Tmax, iters, weight_mode, gamma, st);
    GSS_CASE_K(1) GSS_CASE_K(2) GSS_CASE_K(3) GSS_CASE_K(4) GSS_CASE_K(5) GSS_CASE_K(6) GSS_CASE_K(7) GSS_CASE_K(8)
#undef GSS_CASE_K
    default: return GSS_EUNSUPPORTED;
  }
}

}  // namespace
