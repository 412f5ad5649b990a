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
// costs registers, not time.  The posterior itself (log, exp, normalisation over K) is fp32.
#include "gss_internal.h"

#include <type_traits>

namespace {

constexpr int kWave = 64;

__host__ __device__ constexpr int next_pow2(int x) {
  int p = 1;
  while (p < x) p <<= 1;
  return p;
}

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
// fp64 helpers (no transcendental functions anywhere in the EM loop)
// ----------------------------------------------------------------------------------------------
__device__ __forceinline__ double rcp_f64(double x) {
  double r = __builtin_amdgcn_rcp(x);
  r = fma(fma(-x, r, 1.0), r, r);
  r = fma(fma(-x, r, 1.0), r, r);
  return r;
}

template <int N>
__device__ __forceinline__ double ipow(double x) {
  if constexpr (N == 1) {
    return x;
  } else if constexpr (N % 2 == 0) {
    const double h = ipow<N / 2>(x);
    return h * h;
  } else {
    return x * ipow<N - 1>(x);
  }
}

// Compile-time loop: f(std::integral_constant<int, B>{}), ..., f(std::integral_constant<int, E_ - 1>{}).
template <int B, int E_, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E_) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E_>(f);
  }
}

// Position (row i, column j >= i, part: 0 diagonal, 1 real, 2 imaginary) of packed index idx.
__host__ __device__ constexpr int packed_i(int idx, int D) {
  int i = 0;
  for (int r = 1; r < D; ++r)
    if (idx >= gss_packed_row(r, D)) i = r;
  return i;
}
__host__ __device__ constexpr int packed_j(int idx, int D) {
  const int i = packed_i(idx, D);
  const int off = idx - gss_packed_row(i, D);
  return off == 0 ? i : i + 1 + (off - 1) / 2;
}
__host__ __device__ constexpr int packed_part(int idx, int D) {
  const int off = idx - gss_packed_row(packed_i(idx, D), D);
  return off == 0 ? 0 : 1 + ((off - 1) & 1);
}

// Entry IDX of the Hermitian outer product y y^H in the packed order (see gss_packed_row), fp64.
template <int D, int IDX>
__device__ __forceinline__ double packed_entry(const double (&yr)[D], const double (&yi)[D]) {
  constexpr int i = packed_i(IDX, D), j = packed_j(IDX, D), part = packed_part(IDX, D);
  if constexpr (part == 0) return yr[i] * yr[i] + yi[i] * yi[i];
  else if constexpr (part == 1) return yr[i] * yr[j] + yi[i] * yi[j];   // Re(y_i conj(y_j))
  else return yi[i] * yr[j] - yr[i] * yi[j];                            // Im(y_i conj(y_j))
}

// ----------------------------------------------------------------------------------------------
// Pass kernel for D <= 8 (E = D*D <= 64 packed reals).  One wavefront per workgroup, tiles of 64 frames.
//
// Phase 1 (lane = frame): outer product P = y y^H in fp64; q_k = <coef_k, P> with the class
//   coefficients wave-uniform, read through the scalar path; posterior over the active classes as
//   pi_k / det B_k * q_k^-D in (mantissa, exponent) form, fp64, no log/exp; weights w_k = gamma_k / q_k.
//   P (fp64, column-rotated per row against bank conflicts) and w go to LDS.
// Phase 2 (lane = (frame group tg, entry group eg), 8 x 8): R_k[e] += w_k[t] * P_t[e] in fp64 for the
//   lane's entries e = eg + 8c and frames 4*tg .. 4*tg+3 of a 32-frame half tile.  The half tile keeps
//   the LDS footprint at 16 KB + weights, i.e. two wavefronts per SIMD.  The accumulators stay in
//   registers across the tiles of the chunk.
//
// Grid: blockIdx.x = chunk + C * (f + F * s).  A chunk is `tiles_per_chunk` tiles of 64 frames.
// ----------------------------------------------------------------------------------------------
template <int D, int K, bool FINAL>
__global__ __launch_bounds__(kWave, 2) void em_pass_small(
    const float2* __restrict__ Y, const uint8_t* __restrict__ act, const int32_t* __restrict__ T_len,
    const double* __restrict__ coef, const double* __restrict__ cmant, const int32_t* __restrict__ cexp,
    double* __restrict__ part, double* __restrict__ npart, float* __restrict__ gamma,
    int F, int Tmax, int C, int tiles_per_chunk) {
  constexpr int E = D * D;
  constexpr int EPL = (E + 7) / 8;          // packed entries per lane in phase 2
  constexpr int RS = 64;                    // LDS row stride (doubles); columns rotated by the row index
  constexpr int KP = K | 1;                 // odd row stride of the weight tile
  __shared__ double sP[FINAL ? 1 : 32 * RS];
  __shared__ double sW[FINAL ? 1 : kWave * KP];

  const int lane = threadIdx.x;
  const int chunk = blockIdx.x % C;
  const long sf = blockIdx.x / C;
  const int s = (int)(sf / F);
  const int f = (int)(sf % F);
  int T = T_len ? T_len[s] : Tmax;
  T = T < 0 ? 0 : (T > Tmax ? Tmax : T);
  const int t_end = FINAL ? Tmax : T;       // the final pass also writes the zero padding

  typedef const __attribute__((address_space(4))) double* const_ptr_t;
  const double* __restrict__ cf = coef + sf * (long)(K * E);
  const double* __restrict__ cm = cmant + sf * K;
  const int32_t* __restrict__ ce = cexp + sf * K;

  double acc[EPL][K];
  double nacc[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    nacc[k] = 0.0;
#pragma unroll
    for (int c = 0; c < EPL; ++c) acc[c][k] = 0.0;
  }
  const int tg = lane >> 3, eg = lane & 7;

  const float2* __restrict__ Yrow = Y + sf * (long)Tmax * D;
  const uint8_t* __restrict__ arow = act + (long)s * K * Tmax;

  for (int tile = 0; tile < tiles_per_chunk; ++tile) {
    const int t0 = (chunk * tiles_per_chunk + tile) * kWave;
    if (t0 >= t_end) break;                  // uniform
    const int t = t0 + lane;
    const bool valid = t < T;
    const const_ptr_t cf4 = (const_ptr_t)(uintptr_t)cf;
    int goff = 0;
    asm volatile("" : "+s"(goff));          // opaque (uniform) offset of the first coefficient group

    // ---- phase 1 ----
    double yr[D], yi[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const float2 v = Yrow[(long)(valid ? t : 0) * D + d];     // frame 0 always exists; masked below
      yr[d] = valid ? (double)v.x : 0.0;
      yi[d] = valid ? (double)v.y : 0.0;
    }
    // q_k = <coef_k, P>, P = y y^H generated entry by entry.  The coefficients are loop-invariant and
    // wave-uniform.  Left alone, the compiler hoists all K*E scalar loads out of the tile loop and spills
    // them into vector-register lanes; the empty asm statements below make each group's pointer depend
    // on the previous group's first product and route every partial sum through a fence, which keeps
    // one group's loads next to its use and lets the next group's loads overlap the arithmetic.
    double q[K];
#pragma unroll
    for (int k = 0; k < K; ++k) q[k] = 0.0;
    double n2 = 0.0;
    constexpr int kGroup = 4;
    static_for<0, (E + kGroup - 1) / kGroup>([&](auto GI) {
      constexpr int g = GI.value * kGroup;
      constexpr int ng = (E - g) < kGroup ? (E - g) : kGroup;
      double Pg[ng];
      static_for<0, ng>([&](auto EI) {
        constexpr int e = EI.value;
        Pg[e] = packed_entry<D, g + e>(yr, yi);
        if constexpr (packed_part(g + e, D) == 0) n2 += Pg[e];
      });
      const const_ptr_t cg = cf4 + goff;
      q[0] = fma(cg[0], Pg[0], q[0]);
      int noff = g + kGroup;
      asm volatile("" : "+s"(noff), "+v"(q[0]));
#pragma unroll
      for (int k = 1; k < K; ++k) asm volatile("" : "+v"(q[k]));
#pragma unroll
      for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int e = (k == 0 ? 1 : 0); e < ng; ++e) q[k] = fma(cg[k * E + e], Pg[e], q[k]);
      }
      goff = noff;
    });

    // posterior over the active classes: pi_k / det B_k * q_k^-D with q_k = max(qraw_k / n2c, eps_q)
    const double n2c = fmax(n2, GSS_EPS_NORM_SQ);
    const double qfloor = GSS_EPS_Q * n2c;
    double rq[K], mant[K];
    int ex[K];
    bool a[K];
    int emax = -(1 << 28);
#pragma unroll
    for (int k = 0; k < K; ++k) {
      a[k] = valid && (arow[(long)k * Tmax + (valid ? t : 0)] != 0);
      rq[k] = rcp_f64(fmax(q[k], qfloor));           // 1 / (q_k * n2c): the M-step weight is gamma_k * rq
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
    const double rz = Z > 0.0 ? rcp_f64(Z) : 0.0;
    if (FINAL) {
      if (t < Tmax) {
#pragma unroll
        for (int k = 0; k < K; ++k) gamma[(((long)s * K + k) * F + f) * Tmax + t] = (float)(v[k] * rz);
      }
      continue;
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const double g = v[k] * rz;
      nacc[k] += g;
      sW[lane * KP + k] = g * rq[k];
    }

    // ---- phase 2, two half tiles ----
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      // The 32 lanes of this half rebuild their outer product from y and put it in LDS (cheaper than
      // keeping E doubles alive per lane through the posterior).
#pragma unroll
      for (int d = 0; d < D; ++d) asm volatile("" : "+v"(yr[d]), "+v"(yi[d]));
      if ((lane >> 5) == half) {
        const int row = lane & 31;
        static_for<0, E>([&](auto EI) {
          constexpr int e = EI.value;
          sP[row * RS + ((e + row) & 63)] = packed_entry<D, e>(yr, yi);
          if constexpr ((e & 7) == 7) __builtin_amdgcn_sched_barrier(0);   // bounds the live range of the products
        });
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = 4 * tg + j;              // row in the half tile; its frame is t0 + 32*half + r
        double w[K];
#pragma unroll
        for (int k = 0; k < K; ++k) w[k] = sW[(32 * half + r) * KP + k];
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
          const int e = eg + 8 * c;
          if (e < E) {
            const double p = sP[r * RS + ((e + r) & 63)];
#pragma unroll
            for (int k = 0; k < K; ++k) acc[c][k] = fma(w[k], p, acc[c][k]);
          }
        }
      }
      __syncthreads();
    }
  }
  if (FINAL) return;

  // reduce over the 8 frame groups (lane bits 3..5); lanes 0..7 then hold the chunk's partial sums
#pragma unroll
  for (int k = 0; k < K; ++k) {
#pragma unroll
    for (int c = 0; c < EPL; ++c) {
      double x = acc[c][k];
#pragma unroll
      for (int off = 8; off < kWave; off <<= 1) x += __shfl_xor(x, off, kWave);
      acc[c][k] = x;
    }
    double nv = nacc[k];
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) nv += __shfl_xor(nv, off, kWave);
    if (lane == 0) npart[(sf * C + chunk) * K + k] = nv;
  }
  if (lane < 8) {
#pragma unroll
    for (int c = 0; c < EPL; ++c) {
      const int e = lane + 8 * c;
      if (e < E) {
#pragma unroll
        for (int k = 0; k < K; ++k) part[((sf * C + chunk) * K + k) * (long)E + e] = acc[c][k];
      }
    }
  }
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
    int C, int weight_mode) {
  constexpr int E = D * D;
  __shared__ double sR[K][E];
  __shared__ double sMr[K][D][D], sMi[K][D][D];
  __shared__ double sN[K];
  __shared__ double sDetM[K];
  __shared__ int sDetE[K];

  const long sf = blockIdx.x;
  const int k = threadIdx.x / kWave;
  const int l = threadIdx.x % kWave;

  if (l < E) {
    double r = 0.0;
    for (int c = 0; c < C; ++c) r += part[((sf * C + c) * K + k) * (long)E + l];
    sR[k][l] = r;
  }
  if (l == 0) {
    double n = 0.0;
    for (int c = 0; c < C; ++c) n += npart[(sf * C + c) * K + k];
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
  __syncthreads();

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
    const double rp = 1.0 / piv;
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
    __syncthreads();
    if (on) { sMr[k][i][j] = nr; sMi[k][i][j] = ni; }
    __syncthreads();
  }
  if (l == 0) { sDetM[k] = detm; sDetE[k] = dete; }

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
  __syncthreads();
  if (l == 0) {
    double pi;
    if (weight_mode == 1) {
      double tot = 0.0;
      for (int kk = 0; kk < K; ++kk) tot += sN[kk];
      pi = Nk / fmax(tot, GSS_EPS_N);
    } else {
      pi = 1.0 / (double)K;
    }
    const double c = fmax(pi, GSS_EPS_PI) / sDetM[k];        // pi_k / det B_k = c * 2^-dete
    cmant[sf * K + k] = __builtin_amdgcn_frexp_mant(c);
    cexp[sf * K + k] = __builtin_amdgcn_frexp_exp(c) - sDetE[k];
  }
}

// ----------------------------------------------------------------------------------------------
// Host-side plan and dispatch
// ----------------------------------------------------------------------------------------------
struct EmPlan {
  int C;                 // chunks per (segment, frequency)
  int tiles_per_chunk;   // 64-frame tiles per chunk
  size_t off_coef, off_cm, off_ce, off_part, off_npart, total;
};

EmPlan make_plan(const gss_ctx* ctx, long n_sf, int Tmax, int D, int K) {
  EmPlan p;
  const int tiles = (Tmax + kWave - 1) / kWave;
  // Aim for ~24 single-wave workgroups per compute unit so the tail of a launch is short, but never
  // split finer than one tile per chunk.
  const long target = (long)ctx->num_cu * 24;
  long C = (target + n_sf - 1) / n_sf;
  if (C < 1) C = 1;
  if (C > tiles) C = tiles;
  p.tiles_per_chunk = (int)((tiles + C - 1) / C);
  p.C = (tiles + p.tiles_per_chunk - 1) / p.tiles_per_chunk;
  const size_t E = (size_t)D * D;
  size_t o = 0;
  p.off_coef = o;  o = gss_align_up(o + (size_t)n_sf * K * E * sizeof(double), 256);
  p.off_cm = o;    o = gss_align_up(o + (size_t)n_sf * K * sizeof(double), 256);
  p.off_ce = o;    o = gss_align_up(o + (size_t)n_sf * K * sizeof(int32_t), 256);
  p.off_part = o;  o = gss_align_up(o + (size_t)n_sf * p.C * K * E * sizeof(double), 256);
  p.off_npart = o; o = gss_align_up(o + (size_t)n_sf * p.C * K * sizeof(double), 256);
  p.total = o;
  return p;
}

template <int D, int K>
int run_small(gss_ctx* ctx, const float2* Y, const uint8_t* act, const int32_t* T_len, int S, int F, int Tmax,
              int iters, int weight_mode, float* gamma, hipStream_t st) {
  const long n_sf = (long)S * F;
  const EmPlan p = make_plan(ctx, n_sf, Tmax, D, K);
  int rc = gss_ensure_scratch(ctx, p.total);
  if (rc != GSS_OK) return rc;
  char* base = (char*)ctx->scratch;
  double* coef = (double*)(base + p.off_coef);
  double* cm = (double*)(base + p.off_cm);
  int32_t* ce = (int32_t*)(base + p.off_ce);
  double* part = (double*)(base + p.off_part);
  double* npart = (double*)(base + p.off_npart);

  if ((long)n_sf * p.C > 0x7fffffffL) return GSS_EUNSUPPORTED;
  const dim3 grid((unsigned)(n_sf * p.C));
  hipLaunchKernelGGL(em_init_coef, dim3(1024), dim3(256), 0, st, coef, cm, ce, D, K, n_sf);
  for (int it = 0; it < iters; ++it) {
    hipLaunchKernelGGL((em_pass_small<D, K, false>), grid, dim3(kWave), 0, st, Y, act, T_len, coef, cm, ce, part, npart,
                       (float*)nullptr, F, Tmax, p.C, p.tiles_per_chunk);
    hipLaunchKernelGGL((em_factor_small<D, K>), dim3((unsigned)n_sf), dim3(kWave * K), 0, st, part, npart, coef, cm, ce,
                       ctx->status, p.C, weight_mode);
  }
  hipLaunchKernelGGL((em_pass_small<D, K, true>), grid, dim3(kWave), 0, st, Y, act, T_len, coef, cm, ce,
                     (double*)nullptr, (double*)nullptr, gamma, F, Tmax, p.C, p.tiles_per_chunk);
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

extern "C" int gss_cacgmm_em(gss_ctx* ctx, const float* Y, const uint8_t* activity, const int32_t* T_len,
                             int S, int F, int Tmax, int D, int K, int iters, int weight_mode,
                             float* gamma, void* stream) {
  if (!ctx || !Y || !activity || !gamma) return GSS_EINVAL;
  if (S <= 0 || F <= 0 || Tmax <= 0 || D <= 0 || K <= 0 || iters < 0) return GSS_EINVAL;
  if (weight_mode != 0 && weight_mode != 1) return GSS_EINVAL;
  if (D > GSS_MAX_D || K > GSS_MAX_K) return GSS_EUNSUPPORTED;
  if (hipSetDevice(ctx->device) != hipSuccess) return GSS_EHIP;
  hipStream_t st = (hipStream_t)stream;
  const float2* Yc = (const float2*)Y;
  switch (D) {
#define GSS_CASE_D(DD) \
  case DD: return dispatch_k<DD>(ctx, Yc, activity, T_len, S, F, Tmax, K, iters, weight_mode, gamma, st);
    GSS_CASE_D(1) GSS_CASE_D(2) GSS_CASE_D(3) GSS_CASE_D(4) GSS_CASE_D(5) GSS_CASE_D(6) GSS_CASE_D(7) GSS_CASE_D(8)
#undef GSS_CASE_D
    default: return GSS_EUNSUPPORTED;
  }
}
