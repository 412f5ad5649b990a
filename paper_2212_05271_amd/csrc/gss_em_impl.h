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
// costs registers, not time.  The posterior is fp64 as well, evaluated as pi_k / det B_k * q_k^-D and
// normalised over the classes (no logarithm, no exponential; for D <= 8 every term is a normal double);
// only the gamma that leaves the library is rounded to fp32.
#pragma once

#include "gss_internal.h"

#include "gss_device.h"


namespace {

// ----------------------------------------------------------------------------------------------
// Coefficient initialisation: B = I, log-term 0  (pass 0).
// coef[sf][k][E] packed as gss_packed_row(); cconst[sf][k] = pi_k / det B_k (any common factor cancels in
// the posterior).
// ----------------------------------------------------------------------------------------------
__global__ void em_init_coef(double* __restrict__ coef, double* __restrict__ cconst, int D, int K, long n_sf) {
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
    cconst[i] = 1.0;
  }
}

// ----------------------------------------------------------------------------------------------
// Pass kernel for D <= 8.  Workgroup = kPassWaves wavefronts on the same (segment, frequency); every
// wavefront owns a contiguous range of tiles of 64 frames and a private LDS region, and there is no
// workgroup barrier inside the tile loop.
//
// Class coefficients.  The packed coefficients of B_k^-1 (D * D reals per class) are the same for every
// frame.  They live in vector registers for the whole kernel, 16 per register: lane l of every row of 16
// lanes holds entry 16 r + (l mod 16) of register r, and the FMAs of phase 1 read them with the
// row-broadcast lane selector of the double-precision vector FMA (v_fmac_f64 ... row_newbcast:n takes its
// first factor from lane n of the executing lane's row).  No scalar loads and no LDS traffic in the inner
// loop; D = 8, K = 5 needs 20 register pairs.  When K * ceil(D*D/16) exceeds kResidentRegs the registers
// of one 16-entry block are fetched from an LDS copy of the coefficients at the start of the block instead.
//
// Classes that are not active anywhere in a tile (activity mask, Eq. (5)) have posterior 0 in all of its
// frames and add nothing to any sum: the tile's arithmetic for them is skipped under wave-uniform branches.
//
// Phase 1 (lane = frame): the Hermitian outer product is generated 16 entries at a time in fp64, and
//   q_k = <coef_k, y y^H> takes 16 row-broadcast FMAs per live class and block; posterior over the active
//   classes; weights w_k = gamma_k / q_k.  y (as fp64) and w go to the wavefront's LDS tile.
// Phase 2 (lane = (frame group tg, channel eg), 8 x 8; frames tg, tg+8, ... of the tile): lane type eg = i
//   owns the entries y_i conj(y_b) for b = i+1, i+2, i+3 (mod 8), and either the pair (i, i+4) (i < 4) or
//   the real diagonal entries of channels i and i-4 (i >= 4): 8 real entries per lane, all 64 of the packed
//   Hermitian 8 x 8 matrix over the 8 lane types, the same instructions for every lane except the last two
//   entries.  For its 8 frames per tile a lane reads 5 channels of y and the weights, forms its 8
//   entries exactly and accumulates R_k[e] += w_k * P[e] in fp64.  Channels >= D are zero padding.
//   The accumulators stay in registers across the tiles of the chunk.
//
// Grid: blockIdx.x = chunk + C * (f + F * s).  A chunk is `tiles_per_chunk` tiles of 64 frames.
// ----------------------------------------------------------------------------------------------

// Doubles per frame row of the weight tile in LDS (odd: spreads the rows over the banks).
__host__ __device__ constexpr int weight_stride(int K) { return K | 1; }

// Registers (pairs) of 16 coefficients per class, and how many of them a wavefront keeps resident.
__host__ __device__ constexpr int coef_regs(int D) { return (D * D + 15) / 16; }
constexpr int kResidentRegs = 20;

// Few channels: the lane that owns a frame in phase 1 has all D * D entries of its outer product in registers
// anyway (one block of at most 16), so it adds w_k * P[e] to K * D * D accumulators of its own, and there is no
// LDS tile and no phase 2 (whose 8 x 8 lane layout would run mostly on zero padding below 5 channels).  Used
// when the accumulators fit in registers beside phase 1.  The accumulators are acc[k][e] then (packed order)
// instead of acc[slot n][k], and the sums over the lanes are taken at the end of the pass (transpose_reduce).
constexpr int kDirectMaxAcc = 80;
constexpr int kPrefetchMaxAcc = 64;            // the whole-EM kernel requests the next tile ahead up to this many
__host__ __device__ constexpr bool direct_layout(int D, int K) { return D <= 4 && D * D * K <= kDirectMaxAcc; }
template <int D, int K>
struct PassAcc {
  static constexpr bool direct = direct_layout(D, K);
  static constexpr int rows = direct ? K : 8, cols = direct ? D * D : K;
  using type = double[rows][cols];
};
template <int A, int B>
__device__ __forceinline__ void zero_acc(double (&acc)[A][B]) {
#pragma unroll
  for (int a = 0; a < A; ++a)
#pragma unroll
    for (int b = 0; b < B; ++b) acc[a][b] = 0.0;
}

// The lane's frame of a tile as stored in memory and its activity bits: loaded by the caller of pass_tile
// ahead of time (the whole-EM kernel keeps the one tile of a tiny problem for all iterations, and requests
// the next tile of a streamed problem before it works on the current one).
template <int D>
struct TileRegs {
  float2 y[D];
  unsigned abits;
};
// A lane whose frame lies beyond T reads frame 0 instead (it exists whenever the tile's mask is not empty); its
// activity bits are cleared by pass_tile, not here: nothing in this function waits for a loaded value, so the
// loads of the next tile stay in flight while the current one is worked on.
template <int D>
__device__ __forceinline__ void load_tile_regs(TileRegs<D>& r, const float2* __restrict__ Yrow,
                                               const uint8_t* __restrict__ abrow, int t0, int lane, int T) {
  const int t = t0 + lane;
  const bool valid = t < T;
#pragma unroll
  for (int d = 0; d < D; ++d) r.y[d] = Yrow[(long)(valid ? t : 0) * D + d];
  r.abits = abrow[valid ? t : 0];
}

// One tile of 64 frames starting at frame t0.  `tmask` (wave-uniform) is the tile's activity mask.
//   creg : the resident coefficient registers [K * coef_regs(D)] (used when RESIDENT)
//   sC   : LDS copy of the coefficients, [K * coef_regs(D)][16] doubles (used otherwise)
//   cc   : class constants pi_k / det B_k (wave-uniform)
//   pre  : PRE: the lane's frame, loaded by the caller (nothing is read from Yrow / abrow)
template <int D, int K, bool FINAL, bool RESIDENT, bool PRE = false>
__device__ __forceinline__ void pass_tile(
    const float2* __restrict__ Yrow, const uint8_t* __restrict__ abrow, const double (&creg)[RESIDENT ? K * coef_regs(D) : 1],
    const double* __restrict__ sC, const double (&cc)[K], float* __restrict__ gamma_row /* + k*F*Tmax */,
    uint32_t* __restrict__ status, long gamma_kstride, int T, int Tmax, int t0, int lane, unsigned tmask,
    double* __restrict__ sY, double* __restrict__ sW, typename PassAcc<D, K>::type& acc, double (&nacc)[K],
    const TileRegs<D>* pre = nullptr) {
  constexpr int E = D * D;
  constexpr int R = coef_regs(D);
  constexpr int WS = weight_stride(K);
  constexpr bool DIRECT = PassAcc<D, K>::direct;
  const int tg = lane >> 3, eg = lane & 7;
  tmask &= (1u << K) - 1u;
  const int t = t0 + lane;
  if constexpr (FINAL) {
    // the classes that are not live anywhere in the tile: their zeros
    static_for<0, K>([&](auto KI) {
      constexpr int k = KI.value;
      if (!class_on(tmask, k)) {
        if (t < Tmax) gamma_row[k * gamma_kstride + t] = 0.f;
      }
    });
  }
  if (tmask == 0u) return;                    // no frame of the tile has an active class

  // ---- phase 1: load y ----
  // A lane whose frame lies beyond T reads frame 0 instead (it exists whenever a tile is processed at all, or is
  // padding in the final pass); its activity bits are zero, so its posterior and weights are zero.
  const bool valid = t < T;
  double yr[D], yi[D];
  unsigned abits;
  if constexpr (PRE) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      yr[d] = (double)pre->y[d].x;
      yi[d] = (double)pre->y[d].y;
    }
    abits = valid ? pre->abits : 0u;
  } else {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const float2 v = Yrow[(long)(valid ? t : 0) * D + d];
      yr[d] = (double)v.x;
      yi[d] = (double)v.y;
    }
    abits = abrow[valid ? t : 0];
    abits = valid ? abits : 0u;
  }

  // ---- q_k = <coef_k, y y^H>, 16 entries of the outer product at a time; three partial sums per class (an FMA
  // does not wait for the one before it) ----
  constexpr int NQ = DIRECT ? 2 : 3;          // (fewer registers where the accumulators need them)
  double q[K][3];
  double n2 = 0.0;
  double Pd[DIRECT && !FINAL ? E : 1];        // DIRECT: the frame's packed outer product (one block)
#pragma unroll
  for (int k = 0; k < K; ++k) { q[k][0] = 0.0; q[k][1] = 0.0; q[k][2] = 0.0; }
  static_for<0, R>([&](auto RI) {
    constexpr int r = RI.value;
    constexpr int ng = (E - 16 * r) < 16 ? (E - 16 * r) : 16;
    double c[K];
    if constexpr (!RESIDENT) {
      // this block's coefficient registers, from the LDS copy (requested before the products are formed)
#pragma unroll
      for (int k = 0; k < K; ++k) c[k] = sC[(k * R + r) * 16 + (lane & 15)];
    }
    double P[ng];
    static_for<0, ng>([&](auto EI) {
      constexpr int e = EI.value;
      P[e] = packed_entry<D, 16 * r + e>(yr, yi);
      if constexpr (packed_part(16 * r + e, D) == 0) n2 += P[e];
      if constexpr (DIRECT && !FINAL) Pd[16 * r + e] = P[e];
    });
    static_for<0, K>([&](auto KI) {
      constexpr int k = KI.value;
      if (class_on(tmask, k)) {
        double ck;
        if constexpr (RESIDENT) ck = creg[k * R + r]; else ck = c[k];
        static_for<0, ng>([&](auto EI) {
          constexpr int e = EI.value;
          fma_bcast<e, e == 0>(q[k][e % NQ], ck, P[e]);
        });
      }
    });
  });

  // ---- posterior over the active classes: v_k = pi_k / det B_k * q_k^-D with q_k = max(qraw_k / n2c, eps_q),
  // normalised over k.  For D <= 8 this needs no scaling: B has trace D and eigenvalues >= 1e-6, so
  // 1e-6 <= q <= 1e6 on unit vectors (floored at 1e-10), q^-D lies in [1e-48, 1e80], 1 / det B in
  // [1, 1e42] and pi in [1e-30, 1]: every v_k is a normal double.
  const double n2c = fmax(n2, GSS_EPS_NORM_SQ);
  const double qfloor = GSS_EPS_Q * n2c;
  double rq[K], v[K], Z = 0.0;
  static_for<0, K>([&](auto KI) {
    constexpr int k = KI.value;
    rq[k] = 0.0;
    v[k] = 0.0;
    if (class_on(tmask, k)) {
      rq[k] = rcp_f64_fast(fmax(NQ == 3 ? q[k][0] + q[k][1] + q[k][2] : q[k][0] + q[k][1], qfloor));   // 1 / (q * n2c): the M-step weight is gamma * rq
      const double u = rq[k] * n2c;                             // 1 / q
      const double p = cc[k] * ipow<D>(u);
      v[k] = ((abits >> k) & 1u) ? p : 0.0;
      Z += v[k];
    }
  });
  const double rz = Z > 0.0 ? rcp_f64_fast(Z) : 0.0;
  if constexpr (FINAL) {
    if (valid && !(n2 >= GSS_EPS_NORM_SQ)) atomicOr(status, GSS_STATUS_ZERO_FRAME);
    static_for<0, K>([&](auto KI) {
      constexpr int k = KI.value;
      if (class_on(tmask, k)) {
        if (t < Tmax) gamma_row[k * gamma_kstride + t] = (float)(v[k] * rz);
      }
    });
  } else if constexpr (DIRECT) {
    static_for<0, K>([&](auto KI) {
      constexpr int k = KI.value;
      if (class_on(tmask, k)) {
        const double g = v[k] * rz;
        nacc[k] += g;
        const double w = g * rq[k];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[k][e] = fma(w, Pd[e], acc[k][e]);
      }
    });
  } else {
    // this tile's y and weights go to LDS, then phase 2 runs over it
    store_tile_row<D>(sY + lane * kYStride, yr, yi);
    static_for<0, K>([&](auto KI) {
      constexpr int k = KI.value;
      if (class_on(tmask, k)) {
        const double g = v[k] * rz;
        nacc[k] += g;
        sW[lane * WS + k] = g * rq[k];
      }
    });
    wave_lds_sync();

    // ---- phase 2 ----
    accumulate_tile_masked<K, WS>(sY, sW, tg, eg, tmask, acc);
    wave_lds_sync();
  }
}

// Direct layout: the wavefront's totals of the accumulators acc[k][e] and the class counts nacc[k], written as
// out[k * E + e] and out[K * E + k] (LDS; the caller orders the traffic).  ROWS: the sums of the four rows of 16
// lanes separately, row r at out[r * (K * E + K) + ...], for a caller that adds several such sets anyway (two
// exchange steps less).
template <int D, int K, bool ROWS = false>
__device__ __forceinline__ void store_direct_sums(const typename PassAcc<D, K>::type& acc, const double (&nacc)[K],
                                                  double* __restrict__ out, int lane) {
  constexpr int E = D * D, N = K * E + K;
  double v[N];
#pragma unroll
  for (int k = 0; k < K; ++k) {
#pragma unroll
    for (int e = 0; e < E; ++e) v[k * E + e] = acc[k][e];
    v[K * E + k] = nacc[k];
  }
  transpose_reduce<N, ROWS>(v, lane);
  if constexpr (ROWS) {
    const int n0 = transposed_index(lane & 15);
    double* __restrict__ orow = out + (lane >> 4) * N;
#pragma unroll
    for (int j = 0; j < (N + 15) / 16; ++j)
      if (n0 + 16 * j < N) orow[n0 + 16 * j] = v[j];
  } else {
    const int n0 = transposed_index(lane);
#pragma unroll
    for (int j = 0; j < (N + kWave - 1) / kWave; ++j)
      if (n0 + kWave * j < N) out[n0 + kWave * j] = v[j];
  }
}

template <int D, int K, bool FINAL>
__global__ __launch_bounds__(kWave * kPassWaves, 2) void em_pass_small(
    gss_yview yv, const uint8_t* __restrict__ abyte, const uint32_t* __restrict__ tmask,
    const int32_t* __restrict__ T_len,
    const double* __restrict__ coef, const double* __restrict__ cconst,
    double* __restrict__ part, double* __restrict__ npart, float* __restrict__ gamma, uint32_t* __restrict__ status,
    int F, int Tmax, ChunkMap cmap) {
  constexpr int E = D * D;
  constexpr int R = coef_regs(D);
  constexpr bool RESIDENT = K * R <= kResidentRegs;
  constexpr int WS = weight_stride(K);
  constexpr bool DIRECT = PassAcc<D, K>::direct;        // no tiles in LDS then
  constexpr int kTileDoubles = DIRECT ? 0 : kWave * kYStride + kWave * WS;
  constexpr int kCoefDoubles = RESIDENT ? 0 : K * R * 16;
  // per-wavefront tiles (+ the coefficient copy); the tiles are reused at the end for the cross-wavefront
  // reduction (needs kPassWaves * (64 * K + K); DIRECT: kPassWaves * (K * E + K))
  constexpr int kRedDoubles = DIRECT ? kPassWaves * (K * E + K) : kPassWaves * (64 * K + K);
  constexpr int kTilesDoubles = FINAL ? 2 : (kPassWaves * kTileDoubles > kRedDoubles ? kPassWaves * kTileDoubles : kRedDoubles);
  __shared__ __attribute__((aligned(16))) double lds[kTilesDoubles + kCoefDoubles];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  long sf;
  int chunk, tiles_per_chunk;
  chunk_decode(cmap, blockIdx.x, sf, chunk, tiles_per_chunk);
  const int s = (int)((unsigned)sf / (unsigned)F);
  const int f = (int)((unsigned)sf % (unsigned)F);
  int T;
  const float2* __restrict__ Yrow = y_row(yv, T_len, s, f, D, Tmax, T);
  const int t_end = FINAL ? Tmax : T;       // the final pass also writes the zero padding

  const double* __restrict__ cf = coef + sf * (long)(K * E);
  double* __restrict__ sY = lds + (FINAL ? 0 : wave * kTileDoubles);
  double* __restrict__ sW = sY + (FINAL ? 0 : kWave * kYStride);
  double* __restrict__ sC = lds + kTilesDoubles;

  // The class coefficients: register r of class k holds entries 16 r .. 16 r + 15 of its packed coefficients,
  // entry 16 r + (lane mod 16) in every lane (a lane past the end of the class reads the last entry of the
  // array instead: its value is never used).
  double creg[RESIDENT ? K * R : 1];
  if constexpr (RESIDENT) {
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int e = 16 * r + (lane & 15);
        creg[k * R + r] = cf[k * E + (e < E ? e : E - 1)];
      }
  } else {
    creg[0] = 0.0;
    for (int x = threadIdx.x; x < K * R * 16; x += kWave * kPassWaves) {
      const int k = x / (R * 16), e = x % (R * 16);
      sC[x] = cf[k * E + (e < E ? e : E - 1)];
    }
    __syncthreads();
  }
  // class constants pi_k / det B_k (wave-uniform, read through the scalar path)
  double cc[K];
  {
    typedef const __attribute__((address_space(4))) double* cc_ptr_t;
    const cc_ptr_t ccp = (cc_ptr_t)(uintptr_t)(cconst + sf * K);
#pragma unroll
    for (int k = 0; k < K; ++k) cc[k] = ccp[k];
  }

  typename PassAcc<D, K>::type acc;
  double nacc[K];
  zero_acc(acc);
#pragma unroll
  for (int k = 0; k < K; ++k) nacc[k] = 0.0;
  const uint8_t* __restrict__ abrow = abyte + (long)s * Tmax;
  const int tiles_total = (Tmax + kWave - 1) / kWave;
  // the tile masks are read through the scalar path (they were written by an earlier kernel)
  typedef const __attribute__((address_space(4))) uint32_t* mask_ptr_t;
  const mask_ptr_t tmrow = (mask_ptr_t)(uintptr_t)(tmask + (long)s * tiles_total);
  float* __restrict__ gamma_row = FINAL ? gamma + ((long)s * K * F + f) * Tmax : nullptr;
  const long gamma_kstride = (long)F * Tmax;

  // The chunk's tiles are split into one contiguous range per wavefront (lengths differ by at most one); the
  // assignment depends only on the tile count, so the sums are bitwise reproducible.
  const int tile_lo = chunk * tiles_per_chunk;
  int tile_hi = tile_lo + tiles_per_chunk;
  const int tile_end = (t_end + kWave - 1) / kWave;
  tile_hi = tile_hi < tile_end ? tile_hi : tile_end;
  const int n_tiles = tile_hi > tile_lo ? tile_hi - tile_lo : 0;
  const int my_lo = tile_lo + (n_tiles * wave) / kPassWaves;
  const int my_hi = tile_lo + (n_tiles * (wave + 1)) / kPassWaves;
  for (int tile = my_lo; tile < my_hi; ++tile) {
    pass_tile<D, K, FINAL, RESIDENT>(Yrow, abrow, creg, sC, cc, gamma_row, status, gamma_kstride, T, Tmax, tile * kWave,
                                     lane, tmrow[tile], sY, sW, acc, nacc
                                     );
  }
  if (FINAL) return;

  if constexpr (DIRECT) {
    // every wavefront's totals meet in LDS and are added in the order of the wavefronts
    constexpr int N = K * E + K;
    store_direct_sums<D, K>(acc, nacc, lds + wave * N, lane);
    __syncthreads();
    for (int x = threadIdx.x; x < N; x += kWave * kPassWaves) {
      double sum = lds[x];
#pragma unroll
      for (int w = 1; w < kPassWaves; ++w) sum += lds[w * N + x];
      if (x < K * E) part[(long)blockIdx.x * (K * E) + x] = sum;
      else npart[(long)blockIdx.x * K + (x - K * E)] = sum;
    }
  } else {
    // Reduce over the 8 frame groups and over the wavefronts; write the chunk's packed partial sums and counts.
    reduce_and_store_partials<D, K, true>(acc, nacc, sY, lds, part + (long)blockIdx.x * (K * E),
                                          npart + (long)blockIdx.x * K, lane, wave);
  }
}

// ----------------------------------------------------------------------------------------------
// M-step in one wavefront: the K class matrices B_k = D R_k / N_k from the packed sums sR[K][E] and the class
// counts sN[K] (both in LDS), Hermitised by construction, scaled to trace D, loaded with delta I (identity for a
// class without data), inverted in place; the packed coefficients of B_k^-1 go to sC[K][coef_regs(D) * 16] and
// the class constants pi_k / det B_k to sCC[K] (LDS).  Lane (k, i) = (le / 8, le % 8) holds row i of the matrix
// of class k (8 complex numbers) in registers.  Every lane of the wavefront must be active.  The caller orders
// the LDS traffic before and after (wave_lds_sync).
// ----------------------------------------------------------------------------------------------
template <int D, int K>
__device__ __forceinline__ void factor_classes_in_wave(const double* __restrict__ sR, const double* __restrict__ sN,
                                                       double* __restrict__ sC, double* __restrict__ sCC, int le,
                                                       int weight_mode, uint32_t* __restrict__ status) {
  constexpr int E = D * D;
  constexpr int R = coef_regs(D);
  const int fk = le >> 3, fi = le & 7;                  // class and row of this lane
  // (Written without branches: every lane reads from valid addresses and the unused values are deselected,
  // so that the LDS reads go out together instead of one wait per row entry.)
  const bool on = fk < K && fi < D;
  const int fkc = fk < K ? fk : K - 1, fic = fi < D ? fi : D - 1;
  const double* __restrict__ sRk = sR + fkc * E;
  double ar[8], ai[8];                                  // row fi of class fk
  double tr = 0.0;
#pragma unroll
  for (int d = 0; d < D; ++d) tr += sRk[gss_packed_row(d, D)];
  const double Nk = sN[fkc];
  double Ntot = 0.0;
#pragma unroll
  for (int k = 0; k < K; ++k) Ntot += sN[k];
  // B = D R / max(N, eps); dead if its trace <= eps; else rescaled to trace D (= R * D / tr R)
  // (the test without its division, the scale with a reciprocal: both sit in front of the sweeps)
  const bool dead = !((double)D * tr > GSS_EPS_N * fmax(Nk, GSS_EPS_N));
  const double sc = dead ? 0.0 : (double)D * rcp_f64(tr);
  {
    double v0[8], v1[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      // packed position of entry (min, max) of the row's pair (fi, j): the diagonal entry for j = fi (its
      // neighbour is read along and dropped), Re and Im of the off-diagonal entry otherwise
      const int jc = j < D ? j : D - 1;
      const int lo = fic < jc ? fic : jc, hi = fic < jc ? jc : fic;
      int p = gss_packed_row(lo, D) + (hi > lo ? 1 + 2 * (hi - lo - 1) : 0);
      p = p > E - 2 ? E - 2 : p;                          // the last diagonal entry has no neighbour (D = 1: none at all)
      v0[j] = sRk[hi > lo ? p : gss_packed_row(lo, D)];
      v1[j] = sRk[E > 1 ? p + 1 : 0];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool diag = j == fi;
      const bool use = on && j < D && (diag || !dead);
      double re = v0[j] * sc;
      double im = v1[j] * sc;
      re = diag ? (dead ? 1.0 : re) + GSS_DELTA : re;
      im = diag ? 0.0 : (fi > j ? -im : im);              // lower triangle = conjugate
      ar[j] = use ? re : 0.0;
      ai[j] = use ? im : 0.0;
    }
  }
  // Gauss-Jordan sweeps.  The 8 lanes of a class sit in one half of a row of 16 lanes, so the pivot row
  // reaches them through the lane-permute move (class_row_bcast): nothing goes through LDS, nothing waits.
  // Executed by all lanes (the permute reads lanes, so none may be switched off); lanes without a row carry
  // zeros or garbage that is never stored.  Pivot lane: row scaled by 1 / pivot; the others: row minus
  // (a_ip / pivot) x pivot row -- one expression with the factors selected per lane.
  double det = 1.0;
  static_for<0, D>([&](auto PI) {
    constexpr int p = PI.value;
    double pr[D], pi[D];
#pragma unroll
    for (int j = 0; j < D; ++j) {
      pr[j] = class_row_bcast<p>(ar[j]);
      pi[j] = class_row_bcast<p>(ai[j]);
    }
    double piv = pr[p];
    if (!(piv > 1e-300)) {
      piv = 1e-300;
      if (on && fi == 0) atomicOr(status, GSS_STATUS_NONPD_B);
    }
    det *= piv;
    const double rp = rcp_f64(piv);
    const bool is_piv = fi == p;
    const double fr = ar[p] * rp, fim = ai[p] * rp;      // M_ip / pivot
    const double cr = is_piv ? -rp : fr, ci = is_piv ? 0.0 : fim;
#pragma unroll
    for (int j = 0; j < D; ++j) {
      if (j != p) {
        const double br = is_piv ? 0.0 : ar[j], bi = is_piv ? 0.0 : ai[j];
        ar[j] = br - (cr * pr[j] - ci * pi[j]);
        ai[j] = bi - (cr * pi[j] + ci * pr[j]);
      }
    }
    ar[p] = is_piv ? rp : -fr;
    ai[p] = is_piv ? 0.0 : -fim;
  });
  // packed coefficients of q = sum_i A_ii P_ii + 2 sum_{i<j} (Re A_ij Re P_ij + Im A_ij Im P_ij), A = the
  // Hermitian part of the computed inverse: the coefficient of the pair i < j is A_ij + conj(A_ji), not 2 A_ij.
  // (Rounding leaves the computed inverse slightly non-Hermitian.  For an ill-conditioned B, e.g. a class with
  // fewer frames than channels, whose inverse has entries of 1e6, the quadratic form of the Hermitian part is
  // still good to 1e-10 for the class's own frames, while that of one triangle mirrored is off by up to 1e-4.)
  // The row owners write their upper-triangle entries, then add the conjugates of their lower-triangle entries.
  // (One predicate per entry, the divisions as reciprocals: every lane computes the class constant, one stores.)
  {
    double* __restrict__ sCk = sC + fkc * (R * 16);
    const int prow = gss_packed_row(fic, D);
#pragma unroll
    for (int j = 0; j < D; ++j) {
      const bool diag = j == fi;
      const int pj = diag ? prow : prow + 1 + 2 * (j - fic - 1);
      if (on && j >= fi) {
        sCk[pj] = ar[j];
        if (!diag) sCk[pj + 1] = ai[j];
      }
    }
    wave_lds_sync();
#pragma unroll
    for (int j = 0; j < D; ++j) {
      // entry (fi, j) with j < fi belongs to the pair (j, fi)
      const int pj = gss_packed_row(j, D) + 1 + 2 * (fic - j - 1);
      if (on && j < fi) {
        sCk[pj] += ar[j];
        sCk[pj + 1] -= ai[j];
      }
    }
    const double pi_k = weight_mode == 1 ? Nk * rcp_f64(fmax(Ntot, GSS_EPS_N)) : 1.0 / (double)K;
    const double cck = fmax(pi_k, GSS_EPS_PI) * rcp_f64(det);
    if (on && fi == 0) sCC[fk] = cck;
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
    double* __restrict__ coef, double* __restrict__ cconst, uint32_t* __restrict__ status,
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
    // (the Hermitian part of the computed inverse: A_ij + conj(A_ji), see factor_classes_in_wave)
    if (i == j) {
      cf[gss_packed_row(i, D)] = sMr[k][i][i];
    } else {
      const int p = gss_packed_row(i, D) + 1 + 2 * (j - i - 1);
      cf[p] = sMr[k][i][j] + sMr[k][j][i];
      cf[p + 1] = sMi[k][i][j] - sMi[k][j][i];
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
    cconst[sf * K + k] = ldexp(c, -dete);
  }
}

// Order in which the whole-EM kernel takes the segments of a ragged batch: longest first (equal lengths in index
// order), so that the long problems start early and the launch does not end with a few wavefronts still walking
// the longest segments.  order[rank] = segment; one thread per segment counts the segments ahead of its own.
// Beyond kOrderMaxSegments the order is left as it is (the count is quadratic in the number of segments).
constexpr int kOrderMaxSegments = 4096;
__global__ __launch_bounds__(256) void em_order_segments(gss_yview yv, const int32_t* __restrict__ T_len, int Tmax, int S,
                                                         int32_t* __restrict__ order) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= S) return;
  if (S > kOrderMaxSegments) {
    order[s] = s;
    return;
  }
  const int T = y_frames(yv, T_len, s, Tmax);
  int rank = 0;
  for (int o = 0; o < S; ++o) {
    const int To = y_frames(yv, T_len, o, Tmax);
    rank += (To > T || (To == T && o < s)) ? 1 : 0;
  }
  order[rank] = s;
}

// One pass of a wavefront of the whole-EM kernel over its tiles below tile_end: the one resident tile (NW > 1,
// resident_tiles), or tiles wave, wave + NW, ...  With the direct layout and not too many accumulators there are
// registers to spare, and the frames of the next tile are requested from memory before the current tile is worked on.
template <int D, int K, int NW, bool FINAL, bool RESIDENT, class MaskPtr>
__device__ __forceinline__ void whole_pass(
    const float2* __restrict__ Yrow, const uint8_t* __restrict__ abrow, MaskPtr tmrow,
    const double (&creg)[RESIDENT ? K * coef_regs(D) : 1], const double* __restrict__ sC, const double (&cc)[K],
    float* __restrict__ gamma_row, uint32_t* __restrict__ status, long gamma_kstride, int T, int Tmax, int tile_end,
    bool resident_tiles, int wave, int lane, unsigned my_mask, const TileRegs<D>& pre, double* __restrict__ sY,
    double* __restrict__ sW, typename PassAcc<D, K>::type& acc, double (&nacc)[K]) {
  if constexpr (NW > 1) {
    if (resident_tiles) {
      if (wave < tile_end)
        pass_tile<D, K, FINAL, RESIDENT, true>(Yrow, abrow, creg, sC, cc, gamma_row, status, gamma_kstride, T, Tmax,
                                               wave * kWave, lane, my_mask, sY, sW, acc, nacc, &pre);
      return;
    }
  }
  if constexpr (PassAcc<D, K>::direct && D * D * K <= kPrefetchMaxAcc) {
    constexpr unsigned kmask = (1u << K) - 1u;
    TileRegs<D> cur = pre;                               // (zeros; replaced below when the first tile is live)
    int tile = wave;
    unsigned m = 0u;
    if (tile < tile_end) {
      m = tmrow[tile] & kmask;
      if (m != 0u) load_tile_regs<D>(cur, Yrow, abrow, tile * kWave, lane, T);
    }
    while (tile < tile_end) {
      const int next = tile + NW;
      TileRegs<D> nxt = cur;
      unsigned mn = 0u;
      if (next < tile_end) {
        mn = tmrow[next] & kmask;
        if (mn != 0u) load_tile_regs<D>(nxt, Yrow, abrow, next * kWave, lane, T);
      }
      // (the mask is the same in every lane; the compiler has to be told after the loop-carried copy)
      pass_tile<D, K, FINAL, RESIDENT, true>(Yrow, abrow, creg, sC, cc, gamma_row, status, gamma_kstride, T, Tmax,
                                             tile * kWave, lane, __builtin_amdgcn_readfirstlane(m), sY, sW, acc, nacc,
                                             &cur);
      cur = nxt;
      m = mn;
      tile = next;
    }
  } else {
    for (int tile = wave; tile < tile_end; tile += NW)
      pass_tile<D, K, FINAL, RESIDENT>(Yrow, abrow, creg, sC, cc, gamma_row, status, gamma_kstride, T, Tmax, tile * kWave,
                                       lane, tmrow[tile], sY, sW, acc, nacc);
  }
}

// ----------------------------------------------------------------------------------------------
// Whole-EM kernel: a workgroup of NW wavefronts owns one (segment, frequency) for all iterations.  Per
// iteration every wavefront walks its tiles (pass_tile above), sums its accumulators over the 8 frame groups
// through LDS, and factorises the K class matrices itself, so that the coefficients of the next iteration go
// from LDS straight back into its registers: no partial sums in memory, no second kernel, no launch per
// iteration, and the same fixed summation order on every run.
//   NW = 1: for batches with many problems (segments x frequencies >> resident wavefronts); the wavefront
//           walks all tiles of its problem; nothing is shared between wavefronts.
//   NW = 4: for few problems of few channels.  At most NW tiles (256 frames): wavefront w owns tile w and keeps
//           its frames in registers for all iterations, so an iteration reads nothing from memory.  More tiles:
//           wavefront w walks tiles w, w + NW, ...  The wavefronts' sums meet in LDS (two buffers, used in turn,
//           one barrier per iteration), and every wavefront adds them up in the same order and runs the same
//           factorisation on its own copy.
//
// Factorisation in the wavefront: lane (k, i) = (lane / 8, lane % 8) holds row i of the matrix of class k
// (8 complex numbers) in registers.  B_k = D R_k / N_k is Hermitised by construction (packed sums), scaled
// to trace D and loaded with delta I (identity for a class without data); in-place Gauss-Jordan sweeps
// without pivoting (the pivots of a Hermitian positive-definite matrix are positive; their product is
// det B): the owner of pivot row p publishes it in LDS, the 8 lanes of the class read it back.
// ----------------------------------------------------------------------------------------------
template <int D, int K, int NW>
__global__ __launch_bounds__(kWave * NW, 2) void em_whole_small(
    gss_yview yv, const uint8_t* __restrict__ abyte, const uint32_t* __restrict__ tmask,
    const int32_t* __restrict__ T_len, const int32_t* __restrict__ seg_order, float* __restrict__ gamma,
    uint32_t* __restrict__ status, int F, int Tmax, int iters, int weight_mode) {
  constexpr int E = D * D;
  constexpr int R = coef_regs(D);
  constexpr bool RESIDENT = K * R <= kResidentRegs;
  constexpr int WS = weight_stride(K);
  constexpr bool DIRECT = PassAcc<D, K>::direct;       // no tiles in LDS then
  constexpr int kTileDoubles = DIRECT ? 0 : kWave * kYStride + kWave * WS;
  constexpr int kCoefDoubles = K * R * 16;             // packed coefficients, padded to whole registers
  constexpr int kSumDoubles = K * E + K;               // packed weighted scatter sums, then the class counts
  // The sums, counts and class constants of the M-step live only between the last tile of a pass and the first
  // tile of the next one: they share the tile's region, behind the rows that the reduction of the accumulators
  // uses for staging.  So do the coefficients when they are resident in registers during a pass (otherwise the
  // pass reads them from LDS and they keep a place of their own behind the tile).
  constexpr bool SHARED_MSTEP = !DIRECT;
  constexpr int kSharedDoubles = kSumDoubles + K + (RESIDENT ? kCoefDoubles : 0);
  static_assert(!SHARED_MSTEP || kReduceWaveDoubles + kSharedDoubles <= kTileDoubles,
                "the M-step's buffers must fit behind the reduction rows inside the tile region");
  constexpr int kWaveDoubles = !SHARED_MSTEP ? (kTileDoubles + kCoefDoubles + kSumDoubles + K + 1) / 2 * 2
                               : RESIDENT    ? kTileDoubles
                                             : (kTileDoubles + kCoefDoubles + 1) / 2 * 2;
  constexpr int kShareRows = DIRECT ? 4 : 1;           // sets of sums per wavefront in the shared buffer (NW > 1)
  constexpr int kShareDoubles = NW > 1 ? 2 * NW * kShareRows * kSumDoubles : 0;
  __shared__ __attribute__((aligned(16))) double lds[NW * kWaveDoubles + kShareDoubles];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = NW > 1 ? __builtin_amdgcn_readfirstlane(threadIdx.x / kWave) : 0;
  double* __restrict__ sY = lds + wave * kWaveDoubles;
  double* __restrict__ sW = sY + kWave * kYStride;
  double* __restrict__ sC = sY + (SHARED_MSTEP && RESIDENT ? kReduceWaveDoubles : kTileDoubles);   // [K][R * 16] coefficients of B^-1 for the next pass
  double* __restrict__ sR = SHARED_MSTEP && !RESIDENT ? sY + kReduceWaveDoubles : sC + kCoefDoubles;   // [K][E] packed weighted scatter sums
  double* __restrict__ sN = sR + K * E;                // [K] class counts
  double* __restrict__ sCC = sN + K;                   // [K] class constants pi / det B
  double* __restrict__ sShare = lds + NW * kWaveDoubles;   // [2][NW][kShareRows][kSumDoubles] sums of the wavefronts (NW > 1)
  __shared__ int sSlotAll[NW * kWave];
  int* __restrict__ sSlot = sSlotAll + wave * kWave;       // [64] packed index and sign of the lane's reduction slot

  // workgroup -> (segment, frequency): the segments in the order of seg_order (longest first), if given
  const long sf = blockIdx.x;
  int s = (int)((unsigned)sf / (unsigned)F);
  const int f = (int)((unsigned)sf % (unsigned)F);
  if (seg_order) {
    typedef const __attribute__((address_space(4))) int32_t* order_ptr_t;
    s = ((order_ptr_t)(uintptr_t)seg_order)[s];
  }
  int T;
  const float2* __restrict__ Yrow = y_row(yv, T_len, s, f, D, Tmax, T);
  const uint8_t* __restrict__ abrow = abyte + (long)s * Tmax;
  const int tiles_total = (Tmax + kWave - 1) / kWave;
  typedef const __attribute__((address_space(4))) uint32_t* mask_ptr_t;
  const mask_ptr_t tmrow = (mask_ptr_t)(uintptr_t)(tmask + (long)s * tiles_total);
  float* __restrict__ gamma_row = gamma + ((long)s * K * F + f) * Tmax;
  const long gamma_kstride = (long)F * Tmax;
  const int tiles = (T + kWave - 1) / kWave;

  // NW > 1 and at most NW tiles: this wavefront's one tile: its mask, and the lane's frame in registers.
  // (NW > 1 and more tiles: wavefront w walks tiles w, w + NW, ... like the single wavefront of NW = 1.)
  const bool resident_tiles = NW > 1 && tiles_total <= NW;
  TileRegs<D> pre;
  unsigned my_mask = 0u;
#pragma unroll
  for (int d = 0; d < D; ++d) pre.y[d] = make_float2(0.f, 0.f);
  pre.abits = 0u;
  if constexpr (NW > 1) {
    if (resident_tiles) {
      if (wave < tiles_total) my_mask = tmrow[wave] & ((1u << K) - 1u);
      if (my_mask != 0u) load_tile_regs<D>(pre, Yrow, abrow, wave * kWave, lane, T);   // a frame below T exists
    }
  }

  // pass 0: B = I, uniform weights
  double creg[RESIDENT ? K * R : 1];
  double cc[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    cc[k] = 1.0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int e = 16 * r + (lane & 15);
      double v = 0.0;
#pragma unroll
      for (int d = 0; d < D; ++d)
        if (e == gss_packed_row(d, D)) v = 1.0;
      if constexpr (RESIDENT) creg[k * R + r] = v;
      else if (lane < 16) sC[(k * R + r) * 16 + lane] = v;
    }
  }
  if constexpr (!RESIDENT) {
    creg[0] = 0.0;
    wave_lds_sync();
  }

  // Where the lane's share of the frame-group sums goes: looked up once (the table sits in memory) and parked in
  // LDS.  Everything the end of an iteration derives from the lane number is derived there anew, from a copy of
  // the lane number that the compiler cannot see through: values computed ahead of the iteration loop would be
  // live across the tile loop, where there is no register for them, and come back from scratch memory one
  // dependent load at a time.
  if constexpr (!DIRECT) {
    static constexpr SlotTable kSlots = make_slot_table();
    const int slot = (lane & 7) * 8 + (lane >> 3);     // lane o = 8 n + eg reads back slot (eg, n)
    const int pi0 = kSlots.v[D][slot];
    sSlot[lane] = (pi0 < 0 ? 0x4000 : pi0) | (kSlots.sign[slot] < 0 ? 0x8000 : 0);
  }
  wave_lds_sync();
  for (int it = 0; it < iters; ++it) {
    typename PassAcc<D, K>::type acc;
    double nacc[K];
    zero_acc(acc);
#pragma unroll
    for (int k = 0; k < K; ++k) nacc[k] = 0.0;
    whole_pass<D, K, NW, false, RESIDENT>(Yrow, abrow, tmrow, creg, sC, cc, nullptr, status, gamma_kstride, T, Tmax, tiles,
                                          resident_tiles, wave, lane, my_mask, pre, sY, sW, acc, nacc);

    int le = lane;                                      // the lane number again, opaque
    asm volatile("" : "+v"(le));
    // ---- sums over the 8 frame groups -> packed sR[k][e]; class counts over the lanes -> sN[k] ----
    // (NW > 1: into this wavefront's slot of the shared buffer of this iteration)
    double* __restrict__ sOut = NW > 1 ? sShare + ((it & 1) * NW + wave) * (kShareRows * kSumDoubles) : sR;
    if constexpr (DIRECT) {
      store_direct_sums<D, K, (NW > 1)>(acc, nacc, sOut, le);
      wave_lds_sync();
    } else {
    const int code = sSlot[le];
    const int pidx = (code & 0x4000) ? -1 : (code & 0x3fff);
    const double sgn = (code & 0x8000) ? -1.0 : 1.0;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      double nv = wave_sum_f64(nacc[k]);
      if (le == 0) sOut[K * E + k] = nv;
    }
#pragma unroll
    for (int k0 = 0; k0 < K; k0 += 2) {
#pragma unroll
      for (int c = 0; c < 2; ++c)
        if (k0 + c < K) {
#pragma unroll
          for (int n = 0; n < 8; ++n) sY[(c * 8 + n) * kReduceRow + le] = acc[n][k0 + c];
        }
      wave_lds_sync();
#pragma unroll
      for (int c = 0; c < 2; ++c)
        if (k0 + c < K) {
          double sum = 0.0;
#pragma unroll
          for (int tg = 0; tg < 8; ++tg) sum += sY[(c * 8 + (le >> 3)) * kReduceRow + tg * 8 + (le & 7)];
          if (pidx >= 0) sOut[(k0 + c) * E + pidx] = sgn * sum;
        }
      wave_lds_sync();
    }
    }
    if constexpr (NW > 1) {
      __syncthreads();                                  // every wavefront's sums of this iteration are in place
      const double* __restrict__ all = sShare + (it & 1) * (NW * kShareRows * kSumDoubles);
      for (int e = le; e < kSumDoubles; e += kWave) {
        double sum = all[e];
#pragma unroll
        for (int w = 1; w < NW * kShareRows; ++w) sum += all[w * kSumDoubles + e];
        sR[e] = sum;                                    // sN follows sR
      }
      wave_lds_sync();
    }

    // ---- M-step: B_k from (R_k, N_k), regularised, inverted; coefficients and class constants ----
    factor_classes_in_wave<D, K>(sR, sN, sC, sCC, le, weight_mode, status);
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < K; ++k) {
      {
        // the class constant is the same in every lane: kept in scalar registers across the tile loop
        const double c = sCC[k];
        cc[k] = __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(c)),
                                 __builtin_amdgcn_readfirstlane(__double2loint(c)));
      }
      if constexpr (RESIDENT) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const int e = 16 * r + (le & 15);
          creg[k * R + r] = sC[k * (R * 16) + (e < E ? e : E - 1)];
        }
      }
    }
    wave_lds_sync();
  }

  // final pass: the posteriors = the masks, zero padding included
  {
    typename PassAcc<D, K>::type acc;
    double nacc[K];
    zero_acc(acc);
#pragma unroll
    for (int k = 0; k < K; ++k) nacc[k] = 0.0;
    whole_pass<D, K, NW, true, RESIDENT>(Yrow, abrow, tmrow, creg, sC, cc, gamma_row, status, gamma_kstride, T, Tmax,
                                         tiles_total, resident_tiles, wave, lane, my_mask, pre, sY, sW, acc, nacc);
  }
}

// ----------------------------------------------------------------------------------------------
// Host-side plan and dispatch
// ----------------------------------------------------------------------------------------------
// The whole-EM kernel is used when the batch holds at least this many problems per resident wavefront (so that
// the last, partly filled round of wavefronts is a small part of the run).
constexpr int kWholeMinRounds = 3;
constexpr int kWholeMaxTilesAlways = 5;
constexpr int kWholeQuad = 4;                 // wavefronts per problem of the variant for tiny problems
constexpr int kWholeQuadMaxD = 4;             // ... which is built for up to this many channels
constexpr int kWholeDirectMaxTiles = 25;      // direct layout: tiles in a row up to which a pass costs less than its launches

struct EmPlan {
  ChunkMap acc;          // chunking of the accumulating passes
  ChunkMap fin;          // chunking of the final pass
  long wgs_acc, wgs_fin;
  size_t off_coef, off_cc, off_part, off_npart, off_abyte, off_tmask, off_order, total;
};

EmPlan make_plan(const gss_ctx* ctx, long n_sf, int S, int Tmax, int D, int K, int wgs_per_cu, int wgs_per_cu_fin) {
  EmPlan p;
  const int tiles = (Tmax + kWave - 1) / kWave;
  const int round_up = kPassWaves;                     // a chunk is a whole number of rounds of tiles
  const long slots = (long)ctx->num_cu * wgs_per_cu;
  p.acc = plan_chunk_map(slots, n_sf, tiles, round_up, 0, true);
  p.wgs_acc = chunk_map_wgs(p.acc, n_sf);
  p.fin = plan_chunk_map((long)ctx->num_cu * wgs_per_cu_fin, n_sf, tiles, round_up, 0, true);
  p.wgs_fin = chunk_map_wgs(p.fin, n_sf);
  const size_t E = (size_t)D * D;
  size_t o = 0;
  p.off_coef = o;  o = gss_align_up(o + (size_t)n_sf * K * E * sizeof(double) + 64, 256);
  p.off_cc = o;    o = gss_align_up(o + (size_t)n_sf * K * sizeof(double), 256);
  p.off_part = o;  o = gss_align_up(o + (size_t)p.wgs_acc * K * E * sizeof(double), 256);
  p.off_npart = o; o = gss_align_up(o + (size_t)p.wgs_acc * K * sizeof(double), 256);
  p.off_abyte = o; o = gss_align_up(o + (size_t)S * Tmax, 256);
  p.off_tmask = o; o = gss_align_up(o + (size_t)S * tiles * sizeof(uint32_t), 256);
  p.off_order = o; o = gss_align_up(o + (size_t)S * sizeof(int32_t), 256);
  p.total = o;
  return p;
}

template <int D, int K>
int run_small(gss_ctx* ctx, const gss_yview& Y, const uint8_t* act, const int32_t* T_len, int S, int F, int Tmax,
              int iters, int weight_mode, float* gamma, hipStream_t st) {
  const long n_sf = (long)S * F;
  // resident workgroups per compute unit of the two pass kernels: asked once per instantiation
  static const int wgs_per_cu = resident_wgs(em_pass_small<D, K, false>, kWave * kPassWaves, 2);
  static const int wgs_per_cu_fin = resident_wgs(em_pass_small<D, K, true>, kWave * kPassWaves, 2);
  const EmPlan p = make_plan(ctx, n_sf, S, Tmax, D, K, wgs_per_cu, wgs_per_cu_fin);
  int rc = gss_ensure_scratch(ctx, p.total);
  if (rc != GSS_OK) return rc;
  char* base = (char*)ctx->scratch;
  double* coef = (double*)(base + p.off_coef);
  double* cc = (double*)(base + p.off_cc);
  double* part = (double*)(base + p.off_part);
  double* npart = (double*)(base + p.off_npart);
  uint8_t* abyte = (uint8_t*)(base + p.off_abyte);
  uint32_t* tmask = (uint32_t*)(base + p.off_tmask);
  int32_t* order = (int32_t*)(base + p.off_order);
  const int tiles = (Tmax + kWave - 1) / kWave;

  if ((long)S * tiles > 0x7fffffffL) return GSS_EUNSUPPORTED;
  if (p.wgs_acc > 0x7fffffffL || p.wgs_fin > 0x7fffffffL) return GSS_EUNSUPPORTED;
  const dim3 block(kWave * kPassWaves);
  hipLaunchKernelGGL(em_pack_activity, dim3((unsigned)(S * tiles)), dim3(kWave), 0, st, Y, act, T_len, abyte, tmask, K,
                     Tmax, tiles);
  // Many problems per resident wavefront: one wavefront runs the whole EM of a problem (no partial sums, no
  // factor launches).  Few problems: each one is cut into chunks over several workgroups, one pass and one
  // factor launch per iteration.
  static const int waves_per_cu = resident_wgs(em_whole_small<D, K, 1>, kWave, 8);
  const long whole_min = ctx->em_whole_min_problems >= 0 ? (long)ctx->em_whole_min_problems
                                                         : (long)kWholeMinRounds * ctx->num_cu * waves_per_cu;
  // (Problems of a few tiles also go there whatever their number: two launches per iteration cost more than
  // the whole EM of such a problem in one wavefront.)
  bool whole = n_sf >= whole_min || (ctx->em_whole_min_problems < 0 && tiles <= kWholeMaxTilesAlways);
  // Up to 4 channels there is the variant with four wavefronts per problem.  Tiny problems (at most 4 tiles) that
  // fit the GPU in one round of such workgroups: one tile per wavefront, its frames resident in registers.  With
  // the direct layout (cheap tiles, a launch costs as much as a few dozen of them) also longer problems, the
  // wavefronts taking every fourth tile, when that means fewer tiles in a row than one wavefront per problem
  // (rounds of resident wavefronts x tiles each; the meeting of the four sums counts as one tile); such batches
  // go to the whole-EM kernel unless a pass is so long that the launches per iteration no longer matter.
  bool tiny = false;
  if constexpr (D <= kWholeQuadMaxD) {
    if (ctx->em_whole_min_problems < 0 && n_sf > 0) {
      static const int quads_per_cu = resident_wgs(em_whole_small<D, K, kWholeQuad>, kWave * kWholeQuad, 2);
      const long slots1 = (long)ctx->num_cu * waves_per_cu, slots4 = (long)ctx->num_cu * quads_per_cu;
      const long cost1 = (n_sf + slots1 - 1) / slots1 * tiles;
      const long cost4 = (n_sf + slots4 - 1) / slots4 * ((tiles + kWholeQuad - 1) / kWholeQuad + 1);
      if (tiles <= kWholeQuad && n_sf <= slots4) {
        tiny = whole;
      } else if (direct_layout(D, K) && tiles > 1) {
        const long best = cost4 < cost1 ? cost4 : cost1;
        if (!whole && best <= kWholeDirectMaxTiles) whole = true;
        tiny = whole && cost4 < cost1;
      }
    }
  }
  if (iters > 0 && whole && n_sf <= 0x7fffffffL) {
    // a ragged batch is taken longest segment first
    const int32_t* seg_order = nullptr;
    if (S > 1 && T_len) {
      hipLaunchKernelGGL(em_order_segments, dim3((unsigned)((S + 255) / 256)), dim3(256), 0, st, Y, T_len, Tmax, S, order);
      seg_order = order;
    }
    gss_profile_begin(ctx, 0, st);
    if constexpr (D <= kWholeQuadMaxD) {
      if (tiny)
        hipLaunchKernelGGL((em_whole_small<D, K, kWholeQuad>), dim3((unsigned)n_sf), dim3(kWave * kWholeQuad), 0, st, Y,
                           abyte, tmask, T_len, seg_order, gamma, ctx->status, F, Tmax, iters, weight_mode);
    }
    if (!tiny)
      hipLaunchKernelGGL((em_whole_small<D, K, 1>), dim3((unsigned)n_sf), dim3(kWave), 0, st, Y, abyte, tmask, T_len,
                         seg_order, gamma, ctx->status, F, Tmax, iters, weight_mode);
    gss_profile_end(ctx, 0, st);
    if (hipGetLastError() != hipSuccess) return GSS_EHIP;
    return GSS_OK;
  }
  hipLaunchKernelGGL(em_init_coef, dim3(1024), dim3(256), 0, st, coef, cc, D, K, n_sf);
  for (int it = 0; it < iters; ++it) {
    gss_profile_begin(ctx, 0, st);
    hipLaunchKernelGGL((em_pass_small<D, K, false>), dim3((unsigned)p.wgs_acc), block, 0, st, Y, abyte, tmask, T_len, coef,
                       cc, part, npart, (float*)nullptr, ctx->status, F, Tmax, p.acc);
    gss_profile_end(ctx, 0, st);
    gss_profile_begin(ctx, 1, st);
    hipLaunchKernelGGL((em_factor_small<D, K>), dim3((unsigned)n_sf), dim3(kWave * K), 0, st, part, npart, coef, cc,
                       ctx->status, p.acc, weight_mode);
    gss_profile_end(ctx, 1, st);
  }
  hipLaunchKernelGGL((em_pass_small<D, K, true>), dim3((unsigned)p.wgs_fin), block, 0, st, Y, abyte, tmask, T_len, coef, cc,
                     (double*)nullptr, (double*)nullptr, gamma, ctx->status, F, Tmax, p.fin);
  if (hipGetLastError() != hipSuccess) return GSS_EHIP;
  return GSS_OK;
}

}  // namespace
