// WPE dereverberation (arXiv 2212.05271, Section 2.1: the late reverberation X^tail of the signal model is
// estimated with the weighted-prediction-error algorithm of the works cited there and subtracted) for gfx950.
//
// Per (segment, frequency), with ytilde_t the stack of the L delayed observations y_{t-Delta} .. y_{t-Delta-L+1}
// (N = D L components, component tau*D + d = y_{t-Delta-tau, d}) and x = y at the start, each iteration is
//
//   power  : lambda_t = mean_d |x_{t,d}|^2, floored at 1e-10 of its maximum over the segment's frames
//   cov    : R = sum_t ytilde_t ytilde_t^H / lambda_t  (N x N),  P = sum_t ytilde_t y_t^H / lambda_t  (N x D),
//            fp64 partial sums per chunk of frames
//   solve  : R += 1e-10 tr(R)/N I,  G = R^-1 P
//   apply  : x_t = y_t - G^H ytilde_t  (and lambda for the next iteration, or the complex64 output)
//
// Everything up to the output is fp64: R is built from strongly correlated delayed copies of one signal and
// the solve amplifies rounding errors of the sums by its condition number.
#include "gss_internal.h"

#include "gss_device.h"

namespace {

constexpr int kWpeThreads = 256;

// Staging loop of a workgroup: elements e = first, first + stride, ... below n; load(e) fetches one from memory,
// store(e, v) puts it where it belongs (LDS).  BATCH loads are issued before the first of them is stored: written
// as a plain loop, each element waits out a full memory latency before the next load goes out.
template <int BATCH, class V, class Load, class Store>
__device__ __forceinline__ void staged_copy(int first, int n, int stride, Load load, Store store) {
  for (int e0 = first; e0 < n; e0 += BATCH * stride) {
    V v[BATCH];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int e = e0 + u * stride;
      v[u] = V{};
      if (e < n) v[u] = load(e);
    }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int e = e0 + u * stride;
      if (e < n) store(e, v[u]);
    }
  }
}
constexpr int kWpeTile = 64;                  // frames per LDS window of the covariance kernel
constexpr int kWpeBlockDoubles = 32;          // a 4 x 4 complex block of R or P per lane
constexpr double kWpeEpsPowerRel = 1e-10;
constexpr double kWpeLoadRel = 1e-10;

__device__ inline int clamp_T(const int32_t* T_len, int s, int Tmax) {
  int T = T_len ? T_len[s] : Tmax;
  return T < 0 ? 0 : (T > Tmax ? Tmax : T);
}

// Maximum of lam[0..T) over a workgroup (every thread gets it).  `red` holds one double per wavefront.
__device__ inline double block_max(const double* __restrict__ lam, int T, double* red) {
  double m = 0.0;
  for (int t = threadIdx.x; t < T; t += blockDim.x) m = fmax(m, lam[t]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmax(m, __shfl_xor(m, o));
  const int wave = threadIdx.x / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) red[wave] = m;
  __syncthreads();
  double r = 0.0;
  for (int w = 0; w < (int)(blockDim.x / kWave); ++w) r = fmax(r, red[w]);
  __syncthreads();
  return r;
}

// Frame kernels (power, apply) run one workgroup per block of 256 frames of a (segment, frequency) row.
// Workgroups are dealt to the 8 accelerator dies round-robin by their index; xcd_block() turns the index into
// the logical block so that consecutive logical blocks (the blocks of one row, which share the row's
// prediction coefficients and the frames at their common edge) run on the same die and meet in its L2.
// The grid has 8 * ceil(n / 8) workgroups; the surplus ones get an index >= n and leave.
__device__ __forceinline__ long xcd_block(unsigned b, long per_xcd) { return (long)(b & 7u) * per_xcd + (long)(b >> 3); }

// lambda of the observation itself (first iteration).  The block's frames are read as one contiguous run
// (coalesced), |y|^2 per component goes to LDS, then thread = frame sums its D values in channel order.
// fb = frames per block (256 for D <= 8, 64 for larger arrays: fb * (D | 1) doubles of LDS).
__global__ __launch_bounds__(kWpeThreads) void wpe_power_kernel(const float2* __restrict__ Y, const int32_t* __restrict__ T_len,
                                                                double* __restrict__ lam, int F, int Tmax, int D,
                                                                int blocks_per_sf, long n_blocks, long per_xcd, int fb) {
  __shared__ double sP[kWpeThreads * (GSS_WPE_MAX_D + 1)];
  const long blk = xcd_block(blockIdx.x, per_xcd);
  if (blk >= n_blocks) return;
  const long sf = blk / blocks_per_sf;
  const int t0 = (int)(blk % blocks_per_sf) * fb;
  const int T = clamp_T(T_len, (int)(sf / F), Tmax);
  const int pitch = D | 1;                                // odd: the frames' rows start in different banks
  const float2* __restrict__ Yblk = Y + (sf * Tmax + t0) * D;
  const int n_valid = (T - t0 < fb ? (T - t0 > 0 ? T - t0 : 0) : fb) * D;
  staged_copy<4, float2>(
      threadIdx.x, fb * D, kWpeThreads,
      [&](int e) { return e < n_valid ? Yblk[e] : make_float2(0.f, 0.f); },
      [&](int e, float2 v) {
        const int r = e / D, d = e - r * D;
        const double re = v.x, im = v.y;
        sP[r * pitch + d] = re * re + im * im;
      });
  __syncthreads();
  const int t = t0 + threadIdx.x;
  if ((int)threadIdx.x >= fb || t >= Tmax) return;
  double p = 0.0;
  for (int d = 0; d < D; ++d) p += sP[threadIdx.x * pitch + d];
  lam[sf * Tmax + t] = p / (double)D;
}

// Lane l of the covariance kernel owns one 4 x 4 block: the first nb(nb+1)/2 lanes the blocks (bi >= bj) of
// the lower triangle of R (nb = ceil(N/4)), the next nb * nbd lanes the blocks of P (nbd = ceil(D/4)).
__host__ __device__ inline void wpe_block(int l, int nb, int nbd, int& bi, int& bj, bool& is_p, bool& valid) {
  const int nR = nb * (nb + 1) / 2;
  valid = l < nR + nb * nbd;
  if (l < nR) {                                          // row bi of the triangle holds bi + 1 blocks
    bi = (int)((sqrtf(8.f * (float)l + 1.f) - 1.f) * 0.5f);
    while (bi * (bi + 1) / 2 > l) --bi;
    while ((bi + 1) * (bi + 2) / 2 <= l) ++bi;
    bj = l - bi * (bi + 1) / 2;
    is_p = false;
  } else {
    const int m = valid ? l - nR : 0;
    bi = m / nbd;
    bj = m % nbd;
    is_p = true;
  }
}

// Covariance accumulation.  A workgroup takes a chunk of 64-frame tiles of one (segment, frequency).  Per
// tile the frames t0-Delta-L+1 .. t0+63 are staged in LDS in DESCENDING time order: then ytilde_t is the
// contiguous run of N values that starts Delta frames after frame t, and the values of y_t itself sit right
// before it, whatever D is.  Each lane keeps its 4 x 4 block in registers and adds, frame by frame,
// (w_t a_i) conj(b_j) for its four row values a and four column values b.  Rows >= N and columns >= N (or
// >= D) of the last blocks take whatever follows in the window; nothing ever reads them.
// More than 256 blocks (large arrays): G workgroups per chunk, workgroup g of them takes the blocks
// 256 g .. 256 g + 255 (blockIdx.x = chunk slot * G + g).
// part[(blockIdx.x * 32 + j) * 256 + lane]: the 32 doubles (re, im of entry [i][j'], j = (i*4 + j')*2 + {0,1}).
__global__ __launch_bounds__(kWpeThreads) void wpe_cov_kernel(const float2* __restrict__ Y, const int32_t* __restrict__ T_len,
                                                              const double* __restrict__ lam, double* __restrict__ part,
                                                              int F, int Tmax, int D, int taps, int delay, ChunkMap cmap,
                                                              int win_elems, int G) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  double2* __restrict__ sWin = reinterpret_cast<double2*>(lds_raw);
  double* __restrict__ sWt = reinterpret_cast<double*>(lds_raw + (size_t)win_elems * sizeof(double2));
  double* __restrict__ sRed = sWt + kWpeTile;

  long sf;
  int chunk, tpc;
  chunk_decode(cmap, blockIdx.x / (unsigned)G, sf, chunk, tpc);
  const int T = clamp_T(T_len, (int)(sf / F), Tmax);
  const int N = D * taps;
  const int nb = (N + 3) / 4, nbd = (D + 3) / 4;
  int bi, bj;
  bool is_p, valid;
  wpe_block((int)(blockIdx.x % (unsigned)G) * kWpeThreads + (int)threadIdx.x, nb, nbd, bi, bj, is_p, valid);
  if (!valid) { bi = 0; bj = 0; is_p = false; }
  const int aoff = delay * D + 4 * bi;
  const int boff = is_p ? 4 * bj : delay * D + 4 * bj;

  const double* __restrict__ lrow = lam + sf * Tmax;
  const double floor_l = kWpeEpsPowerRel * block_max(lrow, T, sRed);
  const float2* __restrict__ Yrow = Y + sf * (long)Tmax * D;

  double ar_[4][4], ai_[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) { ar_[i][j] = 0.0; ai_[i][j] = 0.0; }

  const int tile_end = (T + kWpeTile - 1) / kWpeTile;
  const int tile_lo = chunk * tpc;
  const int tile_hi = tile_lo + tpc < tile_end ? tile_lo + tpc : tile_end;
  const int win_frames = kWpeTile + delay + taps - 1;
  for (int tile = tile_lo; tile < tile_hi; ++tile) {
    const int t0 = tile * kWpeTile;
    const int tmax = t0 + kWpeTile - 1;
    __syncthreads();                                    // the previous tile's window is no longer read
    staged_copy<4, float2>(
        threadIdx.x, win_elems, kWpeThreads,
        [&](int e) {
          const int r = e / D, d = e - r * D;
          const int t = tmax - r;
          return (r < win_frames && t >= 0 && t < T) ? Yrow[(long)t * D + d] : make_float2(0.f, 0.f);
        },
        [&](int e, float2 v) { sWin[e] = make_double2((double)v.x, (double)v.y); });   // converted once here, not at every use
    if (threadIdx.x < kWpeTile) {
      const int t = t0 + threadIdx.x;
      double w = 0.0;
      if (t < T) {
        const double l = fmax(lrow[t], floor_l);
        w = l > 0.0 ? 1.0 / l : 0.0;                   // all-zero bin: no weight, R = 0, bin left unchanged
      }
      sWt[threadIdx.x] = w;
    }
    __syncthreads();
#pragma unroll 2
    for (int tt = 0; tt < kWpeTile; ++tt) {
      const int base = (kWpeTile - 1 - tt) * D;
      const double w = sWt[tt];
      double war[4], wai[4], br[4], bim[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const double2 a = sWin[base + aoff + i];
        const double2 b = sWin[base + boff + i];
        war[i] = w * a.x;
        wai[i] = w * a.y;
        br[i] = b.x;
        bim[i] = b.y;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {                   // a conj(b)
          ar_[i][j] = fma(war[i], br[j], fma(wai[i], bim[j], ar_[i][j]));
          ai_[i][j] = fma(wai[i], br[j], fma(-war[i], bim[j], ai_[i][j]));
        }
    }
  }
  double* __restrict__ out = part + (size_t)blockIdx.x * kWpeBlockDoubles * kWpeThreads + threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      out[(size_t)((i * 4 + j) * 2 + 0) * kWpeThreads] = ar_[i][j];
      out[(size_t)((i * 4 + j) * 2 + 1) * kWpeThreads] = ai_[i][j];
    }
}

// Assemble.  Four workgroups per (segment, frequency), one per row of the 4 x 4 blocks: lane l sums row
// blockIdx % 4 of its block over the chunks and writes the four entries, with the Hermitian mirror image,
// into the augmented matrix A[sf] = [R | P] (N rows of N + D complex doubles) in global memory.  (Little
// work per thread on purpose: the kernel is a gather and scatter that wants many wavefronts in flight; one
// workgroup per bin took 85 us on 513 bins, four take 42 us, eight 47 us.)
__global__ __launch_bounds__(kWpeThreads) void wpe_assemble_kernel(const double* __restrict__ part, double2* __restrict__ A,
                                                                   int D, int taps, ChunkMap cmap, int G) {
  const long sf = blockIdx.x / (unsigned)(4 * G);
  const int i = blockIdx.x & 3;
  const int g = (int)(blockIdx.x % (unsigned)(4 * G)) >> 2;      // group of 256 blocks (large arrays: G > 1)
  const int N = D * taps;
  const int W = N + D;
  const int nb = (N + 3) / 4, nbd = (D + 3) / 4;
  int count;
  const long wg0 = chunk_base(cmap, sf, count);
  double2* __restrict__ M = A + sf * (long)N * W;

  int bi, bj;
  bool is_p, valid;
  wpe_block(g * kWpeThreads + (int)threadIdx.x, nb, nbd, bi, bj, is_p, valid);
  if (!valid) return;
  double v[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) v[q] = 0.0;
  for (int c = 0; c < count; ++c) {
    const double* __restrict__ src =
        part + (((size_t)(wg0 + c) * G + g) * kWpeBlockDoubles + (size_t)i * 8) * kWpeThreads + threadIdx.x;
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] += src[(size_t)q * kWpeThreads];
  }
  const int a = 4 * bi + i;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int b = 4 * bj + j;
    const double re = v[2 * j], im = v[2 * j + 1];
    if (is_p) {
      if (a < N && b < D) M[(long)a * W + N + b] = make_double2(re, im);
    } else if (a < N && b < N) {
      if (bi != bj || i > j) {                           // below the diagonal: the entry and its mirror image
        M[(long)a * W + b] = make_double2(re, im);
        M[(long)b * W + a] = make_double2(re, -im);
      } else if (i == j) {
        M[(long)a * W + a] = make_double2(re, 0.0);
      }
    }
  }
}

// Solve.  One workgroup of 16 x 32 threads per (segment, frequency) keeps the whole augmented matrix in
// registers: thread (i, j) owns rows i, i+16, ... and columns j, j+32, j+64.  Gauss-Jordan elimination without
// pivoting (R + loading is Hermitian positive definite) and without scaling the pivot rows: after sweep p
// column p is never touched again, so at the end row a of the right-hand part divided by pivot a is row a of
// G.  Per sweep the owners publish the pivot row and the pivot column of the NEXT sweep in LDS (two
// buffers, one barrier per sweep); every thread reads the values for its rows and columns from there.
// Out: Gc[sf][a][d] = conj(G[a][d]), the coefficient that multiplies ytilde_a in the prediction of y_d.
constexpr int kSolveTR = 16, kSolveTC = 32;
constexpr int kSolveThreads = kSolveTR * kSolveTC;
constexpr int kSolveKR = (GSS_WPE_MAX_N + kSolveTR - 1) / kSolveTR;                      // rows per thread
constexpr int kSolveMC = (GSS_WPE_MAX_N + GSS_WPE_MAX_D + kSolveTC - 1) / kSolveTC;      // columns per thread
constexpr int kSolveRowBuf = kSolveMC * kSolveTC, kSolveColBuf = kSolveKR * kSolveTR;

__global__ __launch_bounds__(kSolveThreads) void wpe_solve_kernel(const double2* __restrict__ A, double2* __restrict__ Gc,
                                                                uint32_t* __restrict__ status, int D, int taps) {
  __shared__ double2 sRow[2][kSolveRowBuf];
  __shared__ double2 sCol[2][kSolveColBuf];
  __shared__ double sPiv[kSolveColBuf];
  const long sf = blockIdx.x;
  const int N = D * taps;
  const int W = N + D;
  const int j = threadIdx.x % kSolveTC, i = threadIdx.x / kSolveTC;
  double2* __restrict__ out = Gc + sf * (long)N * D;
  const double2* __restrict__ M = A + sf * (long)N * W;
  double tre[kSolveKR][kSolveMC], tim[kSolveKR][kSolveMC];
  double tr = 0.0;
#pragma unroll
  for (int k = 0; k < kSolveKR; ++k)
#pragma unroll
    for (int m = 0; m < kSolveMC; ++m) {
      const int r = i + kSolveTR * k, c = j + kSolveTC * m;
      double2 v = make_double2(0.0, 0.0);
      if (r < N && c < W) v = M[r * W + c];
      if (r == c && r < N) tr += v.x;
      tre[k][m] = v.x;
      tim[k][m] = v.y;
    }
  // trace of R: every diagonal entry is held by exactly one thread
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) tr += __shfl_xor(tr, o);
  if ((threadIdx.x & (kWave - 1)) == 0) sPiv[threadIdx.x / kWave] = tr;
  __syncthreads();
  tr = 0.0;
  for (int w = 0; w < kSolveThreads / kWave; ++w) tr += sPiv[w];
  __syncthreads();                                       // sPiv is reused for the pivots
  if (!(tr > 0.0)) {                                     // no frame has a past (or silence): G = 0
    for (int e = threadIdx.x; e < N * D; e += kSolveThreads) out[e] = make_double2(0.0, 0.0);
    return;
  }
  const double load = kWpeLoadRel * tr / (double)N;
#pragma unroll
  for (int k = 0; k < kSolveKR; ++k)
#pragma unroll
    for (int m = 0; m < kSolveMC; ++m)
      if (i + kSolveTR * k == j + kSolveTC * m) tre[k][m] += load;
  // Row q lives in register row q / TR of the threads with i == q % TR, column q in register column q / TC
  // of the threads with j == q % TC: the register index is the same for the whole workgroup, so it is
  // picked with scalar branches and only the lane test is a vector operation.
  auto publish = [&](int q, int buf) {                   // row q and column q of the current matrix
    const int kq = q / kSolveTR, mq = q / kSolveTC;
    const bool row_owner = i == q % kSolveTR, col_owner = j == q % kSolveTC;
#pragma unroll
    for (int k = 0; k < kSolveKR; ++k)
      if (k == kq && row_owner) {
#pragma unroll
        for (int m = 0; m < kSolveMC; ++m) sRow[buf][j + kSolveTC * m] = make_double2(tre[k][m], tim[k][m]);
      }
#pragma unroll
    for (int m = 0; m < kSolveMC; ++m)
      if (m == mq && col_owner) {
#pragma unroll
        for (int k = 0; k < kSolveKR; ++k) sCol[buf][i + kSolveTR * k] = make_double2(tre[k][m], tim[k][m]);
      }
  };
  publish(0, 0);
  __syncthreads();
  const double tiny = 1e-300;
  for (int p = 0; p < N; ++p) {
    const int buf = p & 1;
    double piv = sRow[buf][p].x;
    if (!(piv > tiny)) {
      if (threadIdx.x == 0) atomicOr(status, GSS_STATUS_NONPD_WPE);
      piv = tiny;
    }
    if (threadIdx.x == 0) sPiv[p] = piv;
    const double inv = rcp_f64(piv);
    double fr[kSolveKR], fi[kSolveKR];
    const int kp = p / kSolveTR;
    const double keep = i == p % kSolveTR ? 0.0 : inv;   // the pivot row itself stays
#pragma unroll
    for (int k = 0; k < kSolveKR; ++k) {
      const double2 v = sCol[buf][i + kSolveTR * k];     // rows >= N hold zeros, and so does their column entry
      const double sc = k == kp ? keep : inv;
      fr[k] = v.x * sc;
      fi[k] = v.y * sc;
    }
#pragma unroll
    for (int m = 0; m < kSolveMC; ++m) {
      const int c = j + kSolveTC * m;
      if (c > p && c < W) {
        const double2 pc = sRow[buf][c];
#pragma unroll
        for (int k = 0; k < kSolveKR; ++k) {             // row r -= f_r * row p
          tre[k][m] = fma(-fr[k], pc.x, fma(fi[k], pc.y, tre[k][m]));
          tim[k][m] = fma(-fr[k], pc.y, fma(-fi[k], pc.x, tim[k][m]));
        }
      }
    }
    if (p + 1 < N) publish(p + 1, buf ^ 1);
    __syncthreads();
  }
#pragma unroll
  for (int m = 0; m < kSolveMC; ++m) {
    const int c = j + kSolveTC * m;
    if (c >= N && c < W) {
#pragma unroll
      for (int k = 0; k < kSolveKR; ++k) {
        const int r = i + kSolveTR * k;
        if (r < N) {
          const double inv = rcp_f64(sPiv[r]);
          out[r * D + (c - N)] = make_double2(tre[k][m] * inv, -tim[k][m] * inv);
        }
      }
    }
  }
}

// Apply: lane = frame.  The frames t0-Delta-L+1 .. t0+255 of the bin are staged in LDS (row pitch odd in
// 8-byte units for even D, so that the lanes' rows start in different banks); every lane then subtracts
// the prediction, walking the N components of ytilde_t while the N x D coefficients, which are the same for
// all lanes, come through the scalar path.  FINAL: writes the complex64 output (zero at t >= T); otherwise
// writes lambda_t of the new estimate for the next iteration.
template <int D, bool FINAL>
__global__ __launch_bounds__(kWpeThreads) void wpe_apply_kernel(const float2* __restrict__ Y, const int32_t* __restrict__ T_len,
                                                                const double2* __restrict__ Gc, double* __restrict__ lam,
                                                                float2* __restrict__ X, int F, int Tmax, int taps, int delay,
                                                                int blocks_per_sf, int pitch, long n_blocks, long per_xcd) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  float2* __restrict__ sWin = reinterpret_cast<float2*>(lds_raw);
  const long blk = xcd_block(blockIdx.x, per_xcd);
  if (blk >= n_blocks) return;
  const long sf = blk / blocks_per_sf;
  const int t0 = (int)(blk % blocks_per_sf) * kWpeThreads;
  const int T = clamp_T(T_len, (int)(sf / F), Tmax);
  const int t = t0 + threadIdx.x;
  const int N = D * taps;
  if (t0 >= T) {                                         // nothing valid in this block
    if (t < Tmax) {
      if constexpr (FINAL) {
#pragma unroll
        for (int d = 0; d < D; ++d) X[(sf * Tmax + t) * D + d] = make_float2(0.f, 0.f);
      } else {
        lam[sf * Tmax + t] = 0.0;
      }
    }
    return;
  }
  const int past = delay + taps - 1;                     // frames before t0 that the block needs
  const int rows = kWpeThreads + past;
  const float2* __restrict__ Yrow = Y + sf * (long)Tmax * D;
  staged_copy<6, float2>(
      threadIdx.x, rows * D, kWpeThreads,
      [&](int e) {
        const int r = e / D, d = e - r * D;
        const int tt = t0 - past + r;
        return (tt >= 0 && tt < T) ? Yrow[(long)tt * D + d] : make_float2(0.f, 0.f);
      },
      [&](int e, float2 v) {
        const int r = e / D, d = e - r * D;
        sWin[r * pitch + d] = v;
      });
  __syncthreads();
  double xr[D], xi[D];
  const float2* __restrict__ mine = sWin + (threadIdx.x + past) * pitch;
#pragma unroll
  for (int d = 0; d < D; ++d) { xr[d] = (double)mine[d].x; xi[d] = (double)mine[d].y; }
  typedef const __attribute__((address_space(4))) double* cptr_t;
  const cptr_t g4 = (cptr_t)(uintptr_t)(Gc + sf * (long)N * D);
  if constexpr (D % 2 == 0) {
    // The D coefficients of one component of ytilde are wave-uniform and come through the scalar path; two
    // such rows are resident in SGPRs and the loads of the next row are issued during the arithmetic of the
    // current one (the empty asm statements fix that order: the next row's offset becomes known after the
    // first product of the current row, and every sum passes a fence at the end of the row).  LDS and scalar
    // loads share one counter, so the frame values of the next tap are fetched from LDS along with the first
    // coefficient row of the current tap, one tap ahead.  The pipeline fetches one row past the last one
    // it uses; the coefficient array is followed by padding so that this load stays in bounds.
    double cA[2 * D], cB[2 * D];
    auto fetch = [&](double (&c)[2 * D], int off) {
      const cptr_t cg = g4 + off;
#pragma unroll
      for (int x = 0; x < 2 * D; ++x) c[x] = cg[x];
    };
    float2 vcur[D], vnxt[D];
    {
      const float2* __restrict__ src = mine - delay * pitch;
#pragma unroll
      for (int dp = 0; dp < D; ++dp) vcur[dp] = src[dp];
      int off0 = 0;
      asm volatile("" : "+s"(off0));                    // opaque offset: keeps the loads inside this kernel's loop
      fetch(cA, off0);
    }
    for (int tau = 0; tau < taps; ++tau) {
      const int tn = tau + 1 < taps ? tau + 1 : tau;     // the last tap re-reads its own row (stays in bounds)
      const float2* __restrict__ srcn = mine - (delay + tn) * pitch;
#pragma unroll
      for (int dp = 0; dp < D; ++dp) {
        const double vr = (double)vcur[dp].x, vi = (double)vcur[dp].y;
        double (&cur)[2 * D] = (dp & 1) ? cB : cA;
        double (&nxt)[2 * D] = (dp & 1) ? cA : cB;
        xr[0] = fma(-cur[0], vr, fma(cur[1], vi, xr[0]));  // first use of this row: the wait for its loads lands here
        int noff = (tau * D + dp + 1) * 2 * D;
        asm volatile("" : "+s"(noff), "+v"(xr[0]));
        fetch(nxt, noff);
        if (dp == 0) {
#pragma unroll
          for (int q = 0; q < D; ++q) vnxt[q] = srcn[q];
        }
        xi[0] = fma(-cur[0], vi, fma(-cur[1], vr, xi[0]));
#pragma unroll
        for (int d = 1; d < D; ++d) {                    // x_d -= c[d] * v
          xr[d] = fma(-cur[2 * d], vr, fma(cur[2 * d + 1], vi, xr[d]));
          xi[d] = fma(-cur[2 * d], vi, fma(-cur[2 * d + 1], vr, xi[d]));
        }
#pragma unroll
        for (int d = 0; d < D; ++d) asm volatile("" : "+v"(xr[d]), "+v"(xi[d]));
      }
#pragma unroll
      for (int q = 0; q < D; ++q) vcur[q] = vnxt[q];
    }
  } else {
    for (int tau = 0; tau < taps; ++tau) {
      const float2* __restrict__ src = mine - (delay + tau) * pitch;
#pragma unroll
      for (int dp = 0; dp < D; ++dp) {
        const float2 v = src[dp];
        const double vr = (double)v.x, vi = (double)v.y;
        const cptr_t c = g4 + ((long)(tau * D + dp) * D) * 2;
#pragma unroll
        for (int d = 0; d < D; ++d) {                    // x_d -= c[d] * v
          const double cr = c[2 * d], ci = c[2 * d + 1];
          xr[d] = fma(-cr, vr, fma(ci, vi, xr[d]));
          xi[d] = fma(-cr, vi, fma(-ci, vr, xi[d]));
        }
      }
    }
  }
  if (t >= Tmax) return;
  if constexpr (FINAL) {
    float2* __restrict__ o = X + (sf * Tmax + t) * D;
#pragma unroll
    for (int d = 0; d < D; ++d) o[d] = t < T ? make_float2((float)xr[d], (float)xi[d]) : make_float2(0.f, 0.f);
  } else {
    double p = 0.0;
#pragma unroll
    for (int d = 0; d < D; ++d) p += xr[d] * xr[d] + xi[d] * xi[d];
    lam[sf * Tmax + t] = t < T ? p / (double)D : 0.0;
  }
}

// iters == 0: the output is the input (zero at t >= T).
__global__ __launch_bounds__(kWpeThreads) void wpe_copy_kernel(const float2* __restrict__ Y, const int32_t* __restrict__ T_len,
                                                               float2* __restrict__ X, int F, int Tmax, int D, long n) {
  const long i = (long)blockIdx.x * kWpeThreads + threadIdx.x;
  if (i >= n) return;
  const long frame = i / D;
  const int t = (int)(frame % Tmax);
  const int s = (int)(frame / Tmax / F);
  X[i] = t < clamp_T(T_len, s, Tmax) ? Y[i] : make_float2(0.f, 0.f);
}

// ----------------------------------------------------------------------------------------------
// Large arrays (D > 8 or D * taps > 80; up to D = 32, D * taps = 320).  The covariance, assemble and power
// kernels above serve them too (several groups of 256 blocks); the linear system no longer fits the
// registers of a workgroup, so it is solved in global memory, and the prediction is applied by a kernel
// with a run-time channel count.
// ----------------------------------------------------------------------------------------------
constexpr int kLsNB = 8;                      // columns per panel of the blocked factorisation
constexpr int kLsPitch = kLsNB + 1;           // LDS row pitch of a panel (in double2)
constexpr int kLsThreads = 256;

__device__ __forceinline__ double2 cmul_conj(double2 a, double2 b) {          // a conj(b)
  return make_double2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}

// Solve for large systems: one workgroup per (segment, frequency), the augmented matrix [R | P] stays in
// global memory (it is L2-resident while its workgroup runs).  Blocked right-looking Cholesky factorisation
// R + loading = L L^H, panels of 8 columns staged in LDS; the right-hand side rides along as D extra rows of
// the virtual lower-triangular matrix V (row N + d of V is column d of P, conjugated: V = [R ; P^H]), so that
// after the last panel the storage of P holds L^-1 P.  Then a blocked back substitution L^H G = L^-1 P.
// No pivoting (the matrix is Hermitian positive definite; a pivot <= 1e-300 is floored and flagged).
// Out: Gc[sf][a][d] = conj(G[a][d]).
__global__ __launch_bounds__(kLsThreads) void wpe_solve_large_kernel(double2* __restrict__ A, double2* __restrict__ Gc,
                                                                     uint32_t* __restrict__ status, int D, int taps) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const int N = D * taps;
  const int W = N + D;
  const int R = N + D;                                    // rows of V
  double2* __restrict__ sPanel = reinterpret_cast<double2*>(lds_raw);         // [R][kLsPitch]: V(r, k0 + c)
  double2* __restrict__ sRhs = sPanel + (size_t)R * kLsPitch;                 // [kLsNB][D]: back substitution
  __shared__ double sRed[kLsThreads / kWave];
  const long sf = blockIdx.x;
  double2* __restrict__ M = A + sf * (long)N * W;
  double2* __restrict__ out = Gc + sf * (long)N * D;
  const int tid = threadIdx.x;
  // V(r, c), c < N: r < N: M[r][c]; r >= N: conj(M[c][N + r - N])
  auto ldv = [&](int r, int c) -> double2 {
    if (r < N) return M[(long)r * W + c];
    double2 v = M[(long)c * W + N + (r - N)];
    v.y = -v.y;
    return v;
  };
  auto stv = [&](int r, int c, double2 v) {
    if (r < N) {
      M[(long)r * W + c] = v;
    } else {
      v.y = -v.y;
      M[(long)c * W + N + (r - N)] = v;
    }
  };

  double tr = 0.0;
  for (int a = tid; a < N; a += kLsThreads) tr += M[(long)a * W + a].x;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) tr += __shfl_xor(tr, o);
  if ((tid & (kWave - 1)) == 0) sRed[tid / kWave] = tr;
  __syncthreads();
  tr = 0.0;
  for (int w = 0; w < kLsThreads / kWave; ++w) tr += sRed[w];
  if (!(tr > 0.0)) {                                     // no frame has a past (or silence): G = 0
    for (int e = tid; e < N * D; e += kLsThreads) out[e] = make_double2(0.0, 0.0);
    return;
  }
  const double load = kWpeLoadRel * tr / (double)N;
  const double tiny = 1e-300;

  for (int k0 = 0; k0 < N; k0 += kLsNB) {
    const int bs = N - k0 < kLsNB ? N - k0 : kLsNB;
    // the panel: rows k0 .. R-1, columns k0 .. k0+bs-1 (of the diagonal block only the lower triangle is used)
    for (int e = tid; e < (R - k0) * bs; e += kLsThreads) {
      const int r = k0 + e / bs, c = e % bs;
      double2 v = make_double2(0.0, 0.0);
      if (r >= k0 + c) v = ldv(r, k0 + c);
      if (r == k0 + c) { v.x += load; v.y = 0.0; }
      sPanel[r * kLsPitch + c] = v;
    }
    __syncthreads();
    // Cholesky of the diagonal block, thread (i, j) of the first 64
    {
      const int i = tid >> 3, j = tid & 7;
      const bool on = tid < 64 && i < bs && j < bs;
      for (int p = 0; p < bs; ++p) {
        if (tid == 0) {
          double d = sPanel[(k0 + p) * kLsPitch + p].x;
          if (!(d > tiny)) {
            d = tiny;
            atomicOr(status, GSS_STATUS_NONPD_WPE);
          }
          sPanel[(k0 + p) * kLsPitch + p] = make_double2(sqrt(d), 0.0);
        }
        __syncthreads();
        if (on && j == p && i > p) {
          const double inv = 1.0 / sPanel[(k0 + p) * kLsPitch + p].x;
          double2 v = sPanel[(k0 + i) * kLsPitch + p];
          sPanel[(k0 + i) * kLsPitch + p] = make_double2(v.x * inv, v.y * inv);
        }
        __syncthreads();
        if (on && j > p && i >= j) {
          const double2 a = sPanel[(k0 + i) * kLsPitch + p], b = sPanel[(k0 + j) * kLsPitch + p];
          const double2 m = cmul_conj(a, b);
          double2 v = sPanel[(k0 + i) * kLsPitch + j];
          sPanel[(k0 + i) * kLsPitch + j] = make_double2(v.x - m.x, v.y - m.y);
        }
        __syncthreads();
      }
    }
    // rows below the block: x L_kk^H = a, one row per thread; the factor goes back to memory
    for (int r = k0 + tid; r < R; r += kLsThreads) {
      if (r < k0 + bs) {
        for (int c = 0; c <= r - k0; ++c) stv(r, k0 + c, sPanel[r * kLsPitch + c]);
        continue;
      }
      double2 x[kLsNB];
#pragma unroll
      for (int c = 0; c < kLsNB; ++c) {
        if (c < bs) {
          double2 acc = sPanel[r * kLsPitch + c];
#pragma unroll
          for (int m = 0; m < kLsNB; ++m)
            if (m < c) {
              const double2 t = cmul_conj(x[m], sPanel[(k0 + c) * kLsPitch + m]);
              acc.x -= t.x;
              acc.y -= t.y;
            }
          const double inv = 1.0 / sPanel[(k0 + c) * kLsPitch + c].x;
          x[c] = make_double2(acc.x * inv, acc.y * inv);
        } else {
          x[c] = make_double2(0.0, 0.0);
        }
      }
#pragma unroll
      for (int c = 0; c < kLsNB; ++c)
        if (c < bs) {
          sPanel[r * kLsPitch + c] = x[c];
          stv(r, k0 + c, x[c]);
        }
    }
    __syncthreads();
    // trailing update: V(r, c) -= sum_m L(r, m) conj(L(c, m)) for k0+bs <= c < N, c <= r < R
    const int c_lo = k0 + bs;
    const int ncols = N - c_lo;
    if (ncols > 0) {
      const int nrows = R - c_lo;
      // four entries per thread and step: their loads are issued together (the entries of different threads and
      // steps are distinct, which the compiler cannot know)
      constexpr int U = 4;
      for (int e0 = tid; e0 < nrows * ncols; e0 += U * kLsThreads) {
        int rr[U], cc[U];
        bool on[U];
        double2 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int e = e0 + u * kLsThreads;
          rr[u] = c_lo + e / ncols;
          cc[u] = c_lo + e % ncols;
          on[u] = e < nrows * ncols && cc[u] <= rr[u];
          v[u] = make_double2(0.0, 0.0);
          if (on[u]) v[u] = ldv(rr[u], cc[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (!on[u]) continue;
          double2 acc = make_double2(0.0, 0.0);
#pragma unroll
          for (int m = 0; m < kLsNB; ++m)
            if (m < bs) {
              const double2 t = cmul_conj(sPanel[rr[u] * kLsPitch + m], sPanel[cc[u] * kLsPitch + m]);
              acc.x += t.x;
              acc.y += t.y;
            }
          v[u].x -= acc.x;
          v[u].y -= acc.y;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (on[u]) stv(rr[u], cc[u], v[u]);
      }
    }
    __syncthreads();
  }

  // back substitution L^H G = Z with Z = L^-1 P in the storage of P (M[c][N + d]); G overwrites it
  const int last = (N - 1) / kLsNB * kLsNB;
  for (int k0 = last; k0 >= 0; k0 -= kLsNB) {
    const int bs = N - k0 < kLsNB ? N - k0 : kLsNB;
    for (int e = tid; e < bs * bs; e += kLsThreads) {     // L_kk (lower triangle)
      const int i = e / bs, j = e % bs;
      if (j <= i) sPanel[i * kLsPitch + j] = M[(long)(k0 + i) * W + k0 + j];
    }
    for (int e = tid; e < bs * D; e += kLsThreads) sRhs[e] = M[(long)(k0 + e / D) * W + N + e % D];
    __syncthreads();
    if (tid < D) {                                         // one right-hand side per thread
      for (int c = bs - 1; c >= 0; --c) {
        double2 acc = sRhs[c * D + tid];
        for (int m = c + 1; m < bs; ++m) {                 // conj(L(m, c)) g_m
          const double2 lmc = sPanel[m * kLsPitch + c], g = sRhs[m * D + tid];
          acc.x -= lmc.x * g.x + lmc.y * g.y;
          acc.y -= lmc.x * g.y - lmc.y * g.x;
        }
        const double inv = 1.0 / sPanel[c * kLsPitch + c].x;
        acc.x *= inv;
        acc.y *= inv;
        sRhs[c * D + tid] = acc;
        M[(long)(k0 + c) * W + N + tid] = acc;
      }
    }
    __syncthreads();
    // rows above the block: Z(r, d) -= sum_m conj(L(k0 + m, r)) G(k0 + m, d)
    for (int e = tid; e < k0 * D; e += kLsThreads) {
      const int r = e % k0, d = e / k0;
      double2 acc = make_double2(0.0, 0.0);
      for (int m = 0; m < bs; ++m) {
        const double2 lmr = M[(long)(k0 + m) * W + r], g = sRhs[m * D + d];
        acc.x += lmr.x * g.x + lmr.y * g.y;
        acc.y += lmr.x * g.y - lmr.y * g.x;
      }
      double2 z = M[(long)r * W + N + d];
      M[(long)r * W + N + d] = make_double2(z.x - acc.x, z.y - acc.y);
    }
    __syncthreads();
  }
  for (int e = tid; e < N * D; e += kLsThreads) {
    const double2 g = M[(long)(e / D) * W + N + e % D];
    out[e] = make_double2(g.x, -g.y);
  }
}

// Apply for large arrays: lane = frame, fb frames per workgroup (+ the needed past) staged in LDS as they
// came; a lane holds all D outputs (up to 32) and walks the D * taps components of ytilde_t; the
// coefficients are the same for all lanes and come through the scalar path, 8 outputs at a time.  A row of
// coefficients is read in whole groups of 8: the last group of a row may reach into the next row (or, at the
// very end of the array, into its padding); those values only enter accumulators that are never stored.
template <bool FINAL>
__global__ __launch_bounds__(kWpeThreads) void wpe_apply_large_kernel(const float2* __restrict__ Y, const int32_t* __restrict__ T_len,
                                                                      const double2* __restrict__ Gc, double* __restrict__ lam,
                                                                      float2* __restrict__ X, int F, int Tmax, int D, int taps,
                                                                      int delay, int blocks_per_sf, int pitch, int fb,
                                                                      long n_blocks, long per_xcd) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  float2* __restrict__ sWin = reinterpret_cast<float2*>(lds_raw);
  const long blk = xcd_block(blockIdx.x, per_xcd);
  if (blk >= n_blocks) return;
  const long sf = blk / blocks_per_sf;
  const int t0 = (int)(blk % blocks_per_sf) * fb;
  const int T = clamp_T(T_len, (int)(sf / F), Tmax);
  const int t = t0 + threadIdx.x;
  const bool mine_on = (int)threadIdx.x < fb && t < Tmax;
  const int N = D * taps;
  if (t0 >= T) {                                         // nothing valid in this block
    if (mine_on) {
      if constexpr (FINAL) {
        for (int d = 0; d < D; ++d) X[(sf * Tmax + t) * D + d] = make_float2(0.f, 0.f);
      } else {
        lam[sf * Tmax + t] = 0.0;
      }
    }
    return;
  }
  const int past = delay + taps - 1;
  const int rows = fb + past;
  const float2* __restrict__ Yrow = Y + sf * (long)Tmax * D;
  staged_copy<6, float2>(
      threadIdx.x, rows * D, kWpeThreads,
      [&](int e) {
        const int r = e / D, d = e - r * D;
        const int tt = t0 - past + r;
        return (tt >= 0 && tt < T) ? Yrow[(long)tt * D + d] : make_float2(0.f, 0.f);
      },
      [&](int e, float2 v) {
        const int r = e / D, d = e - r * D;
        sWin[r * pitch + d] = v;
      });
  __syncthreads();
  if ((int)threadIdx.x >= fb) return;
  constexpr int DM = 32;
  double xr[DM], xi[DM];
  const float2* __restrict__ mine = sWin + (threadIdx.x + past) * pitch;
#pragma unroll
  for (int d = 0; d < DM; ++d) {
    xr[d] = 0.0;
    xi[d] = 0.0;
    if (d < D) {
      xr[d] = (double)mine[d].x;
      xi[d] = (double)mine[d].y;
    }
  }
  typedef const __attribute__((address_space(4))) double* cptr_t;
  const cptr_t g4 = (cptr_t)(uintptr_t)(Gc + sf * (long)N * D);
  for (int tau = 0; tau < taps; ++tau) {
    const float2* __restrict__ src = mine - (delay + tau) * pitch;
    for (int dp = 0; dp < D; ++dp) {
      const float2 v = src[dp];
      const double vr = (double)v.x, vi = (double)v.y;
      const cptr_t c = g4 + ((long)(tau * D + dp) * D) * 2;
      static_for<0, DM / 8>([&](auto GI) {
        constexpr int g = GI.value;
        if (8 * g < D) {
#pragma unroll
          for (int d = 0; d < 8; ++d) {                  // x_d -= c[d] * v
            const double cr = c[2 * (8 * g + d)], ci = c[2 * (8 * g + d) + 1];
            xr[8 * g + d] = fma(-cr, vr, fma(ci, vi, xr[8 * g + d]));
            xi[8 * g + d] = fma(-cr, vi, fma(-ci, vr, xi[8 * g + d]));
          }
        }
      });
    }
  }
  if (t >= Tmax) return;
  if constexpr (FINAL) {
    float2* __restrict__ o = X + (sf * Tmax + t) * D;
#pragma unroll
    for (int d = 0; d < DM; ++d)
      if (d < D) o[d] = t < T ? make_float2((float)xr[d], (float)xi[d]) : make_float2(0.f, 0.f);
  } else {
    double p = 0.0;
#pragma unroll
    for (int d = 0; d < DM; ++d)
      if (d < D) p += xr[d] * xr[d] + xi[d] * xi[d];
    lam[sf * Tmax + t] = t < T ? p / (double)D : 0.0;
  }
}

int run_wpe_large(gss_ctx* ctx, const float2* Y, const int32_t* T_len, int S, int F, int Tmax, int D, int taps, int delay,
                  int iters, float2* X, hipStream_t st) {
  const long n_sf = (long)S * F;
  const int N = D * taps;
  const int W = N + D;
  const int tiles = (Tmax + kWpeTile - 1) / kWpeTile;
  const int nb = (N + 3) / 4, nbd = (D + 3) / 4;
  const int G = (nb * (nb + 1) / 2 + nb * nbd + kWpeThreads - 1) / kWpeThreads;
  const int win_elems = (kWpeTile + delay + taps) * D + 8;
  const int cov_lds = (int)(win_elems * sizeof(double2) + (kWpeTile + kWpeThreads / kWave) * sizeof(double));
  const int fb_apply = D > 24 ? 128 : 256, fb_power = 64;
  const int apitch = D | 1;
  const int apply_lds = (int)((size_t)(fb_apply + delay + taps - 1) * apitch * sizeof(float2));
  const int solve_lds = (int)(((size_t)(N + D) * kLsPitch + (size_t)kLsNB * D) * sizeof(double2));
  if (apply_lds > 64 * 1024 || cov_lds > 64 * 1024 || solve_lds > 64 * 1024) return GSS_EUNSUPPORTED;
  if (hipFuncSetAttribute((const void*)wpe_solve_large_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, solve_lds) !=
          hipSuccess ||
      hipFuncSetAttribute((const void*)wpe_apply_large_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                          apply_lds) != hipSuccess ||
      hipFuncSetAttribute((const void*)wpe_apply_large_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                          apply_lds) != hipSuccess ||
      hipFuncSetAttribute((const void*)wpe_cov_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, cov_lds) != hipSuccess)
    return GSS_EHIP;
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, wpe_cov_kernel, kWpeThreads, (size_t)cov_lds) != hipSuccess ||
      per_cu < 1)
    per_cu = 1;
  // G workgroups per chunk: the chunks are planned for a G-th of the resident workgroups
  long slots = (long)ctx->num_cu * per_cu / G;
  if (slots < 1) slots = 1;
  const ChunkMap cmap = plan_chunk_map(slots, n_sf, tiles, 1, 0, true);
  const long wgs = chunk_map_wgs(cmap, n_sf);
  const long bps_apply = (Tmax + fb_apply - 1) / fb_apply, bps_power = (Tmax + fb_power - 1) / fb_power;
  if (wgs * G > 0x7fffffffL || n_sf * bps_power + 8 > 0x7fffffffL || n_sf * 4 * G > 0x7fffffffL) return GSS_EUNSUPPORTED;

  size_t o = 0;
  const size_t off_lam = o;  o = gss_align_up(o + (size_t)n_sf * Tmax * sizeof(double), 256);
  const size_t off_g = o;    o = gss_align_up(o + (size_t)n_sf * N * D * sizeof(double2) + 1024, 256);   // + read-ahead padding
  const size_t off_part = o; o = gss_align_up(o + (size_t)wgs * G * kWpeBlockDoubles * kWpeThreads * sizeof(double), 256);
  const size_t off_a = o;    o = gss_align_up(o + (size_t)n_sf * N * W * sizeof(double2), 256);
  const int rc = gss_ensure_scratch(ctx, o);
  if (rc != GSS_OK) return rc;
  char* base = (char*)ctx->scratch;
  double* lam = (double*)(base + off_lam);
  double2* Gc = (double2*)(base + off_g);
  double* part = (double*)(base + off_part);
  double2* A = (double2*)(base + off_a);

  const dim3 block(kWpeThreads);
  const long nb_power = n_sf * bps_power, px_power = (nb_power + 7) / 8;
  const long nb_apply = n_sf * bps_apply, px_apply = (nb_apply + 7) / 8;
  hipLaunchKernelGGL(wpe_power_kernel, dim3((unsigned)(8 * px_power)), block, 0, st, Y, T_len, lam, F, Tmax, D,
                     (int)bps_power, nb_power, px_power, fb_power);
  for (int it = 0; it < iters; ++it) {
    gss_profile_begin(ctx, 2, st);
    hipLaunchKernelGGL(wpe_cov_kernel, dim3((unsigned)(wgs * G)), block, cov_lds, st, Y, T_len, lam, part, F, Tmax, D, taps,
                       delay, cmap, win_elems, G);
    gss_profile_end(ctx, 2, st);
    hipLaunchKernelGGL(wpe_assemble_kernel, dim3((unsigned)(n_sf * 4 * G)), block, 0, st, part, A, D, taps, cmap, G);
    hipLaunchKernelGGL(wpe_solve_large_kernel, dim3((unsigned)n_sf), dim3(kLsThreads), solve_lds, st, A, Gc, ctx->status, D,
                       taps);
    if (it + 1 < iters)
      hipLaunchKernelGGL((wpe_apply_large_kernel<false>), dim3((unsigned)(8 * px_apply)), block, apply_lds, st, Y, T_len, Gc,
                         lam, X, F, Tmax, D, taps, delay, (int)bps_apply, apitch, fb_apply, nb_apply, px_apply);
    else
      hipLaunchKernelGGL((wpe_apply_large_kernel<true>), dim3((unsigned)(8 * px_apply)), block, apply_lds, st, Y, T_len, Gc,
                         lam, X, F, Tmax, D, taps, delay, (int)bps_apply, apitch, fb_apply, nb_apply, px_apply);
  }
  if (hipGetLastError() != hipSuccess) return GSS_EHIP;
  return GSS_OK;
}

template <int D>
int run_wpe(gss_ctx* ctx, const float2* Y, const int32_t* T_len, int S, int F, int Tmax, int taps, int delay, int iters,
            float2* X, hipStream_t st) {
  const long n_sf = (long)S * F;
  const int N = D * taps;
  const int W = N + D;
  const int tiles = (Tmax + kWpeTile - 1) / kWpeTile;
  // covariance kernel: window of 64 + delay + taps - 1 frames, plus room for the overrun of the last blocks
  const int win_elems = (kWpeTile + delay + taps) * D + 8;
  const int cov_lds = (int)(win_elems * sizeof(double2) + (kWpeTile + kWpeThreads / kWave) * sizeof(double));
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, wpe_cov_kernel, kWpeThreads, (size_t)cov_lds) != hipSuccess ||
      per_cu < 1)
    per_cu = 1;
  const ChunkMap cmap = plan_chunk_map((long)ctx->num_cu * per_cu, n_sf, tiles, 1, 0, true);
  const long wgs = chunk_map_wgs(cmap, n_sf);
  const long blocks_per_sf = (Tmax + kWpeThreads - 1) / kWpeThreads;
  if (wgs > 0x7fffffffL || n_sf * blocks_per_sf + 8 > 0x7fffffffL || n_sf * 4 > 0x7fffffffL) return GSS_EUNSUPPORTED;
  // apply kernel: row pitch odd for even D
  const int apitch = D | 1;
  const int apply_lds = (int)((size_t)(kWpeThreads + delay + taps - 1) * apitch * sizeof(float2));
  if (apply_lds > 64 * 1024 || cov_lds > 64 * 1024) return GSS_EUNSUPPORTED;

  size_t o = 0;
  const size_t off_lam = o;  o = gss_align_up(o + (size_t)n_sf * Tmax * sizeof(double), 256);
  const size_t off_g = o;    o = gss_align_up(o + (size_t)n_sf * N * D * sizeof(double2) + 256, 256);   // + read-ahead padding
  const size_t off_part = o; o = gss_align_up(o + (size_t)wgs * kWpeBlockDoubles * kWpeThreads * sizeof(double), 256);
  const size_t off_a = o;    o = gss_align_up(o + (size_t)n_sf * N * W * sizeof(double2), 256);
  const int rc = gss_ensure_scratch(ctx, o);
  if (rc != GSS_OK) return rc;
  char* base = (char*)ctx->scratch;
  double* lam = (double*)(base + off_lam);
  double2* Gc = (double2*)(base + off_g);
  double* part = (double*)(base + off_part);
  double2* A = (double2*)(base + off_a);

  const dim3 block(kWpeThreads);
  const long n_blocks = n_sf * blocks_per_sf, per_xcd = (n_blocks + 7) / 8;
  const dim3 frame_grid((unsigned)(8 * per_xcd));
  hipLaunchKernelGGL(wpe_power_kernel, frame_grid, block, 0, st, Y, T_len, lam, F, Tmax, D, (int)blocks_per_sf, n_blocks,
                     per_xcd, kWpeThreads);
  for (int it = 0; it < iters; ++it) {
    gss_profile_begin(ctx, 2, st);
    hipLaunchKernelGGL(wpe_cov_kernel, dim3((unsigned)wgs), block, cov_lds, st, Y, T_len, lam, part, F, Tmax, D, taps, delay,
                       cmap, win_elems, 1);
    gss_profile_end(ctx, 2, st);
    hipLaunchKernelGGL(wpe_assemble_kernel, dim3((unsigned)(n_sf * 4)), block, 0, st, part, A, D, taps, cmap, 1);
    hipLaunchKernelGGL(wpe_solve_kernel, dim3((unsigned)n_sf), dim3(kSolveThreads), 0, st, A, Gc, ctx->status, D, taps);
    if (it + 1 < iters)
      hipLaunchKernelGGL((wpe_apply_kernel<D, false>), frame_grid, block, apply_lds, st, Y, T_len, Gc, lam, X, F, Tmax, taps,
                         delay, (int)blocks_per_sf, apitch, n_blocks, per_xcd);
    else
      hipLaunchKernelGGL((wpe_apply_kernel<D, true>), frame_grid, block, apply_lds, st, Y, T_len, Gc, lam, X, F, Tmax, taps,
                         delay, (int)blocks_per_sf, apitch, n_blocks, per_xcd);
  }
  if (hipGetLastError() != hipSuccess) return GSS_EHIP;
  return GSS_OK;
}

}  // namespace

extern "C" int gss_wpe(gss_ctx* ctx, const float* Y, const int32_t* T_len, int S, int F, int Tmax, int D,
                       int taps, int delay, int iters, float* X, void* stream) {
  if (!ctx || !Y || !X || Y == X) return GSS_EINVAL;
  if (S <= 0 || F <= 0 || Tmax <= 0 || D <= 0 || taps <= 0 || delay <= 0 || iters < 0) return GSS_EINVAL;
  if (D > GSS_WPE_LARGE_MAX_D || (long)D * taps > GSS_WPE_LARGE_MAX_N || delay > 64) return GSS_EUNSUPPORTED;
  bool small = D <= GSS_WPE_MAX_D && (long)D * taps <= GSS_WPE_MAX_N;
  if (small) {
    const int N = D * taps, nb = (N + 3) / 4, nbd = (D + 3) / 4;
    if (nb * (nb + 1) / 2 + nb * nbd > kWpeThreads) small = false;               // more than one block per lane
  }
  if (hipSetDevice(ctx->device) != hipSuccess) return GSS_EHIP;
  hipStream_t st = (hipStream_t)stream;
  const float2* Yc = (const float2*)Y;
  float2* Xc = (float2*)X;
  if (iters == 0) {
    const long n = (long)S * F * Tmax * D;
    const long blocks = (n + kWpeThreads - 1) / kWpeThreads;
    if (blocks > 0x7fffffffL) return GSS_EUNSUPPORTED;
    hipLaunchKernelGGL(wpe_copy_kernel, dim3((unsigned)blocks), dim3(kWpeThreads), 0, st, Yc, T_len, Xc, F, Tmax, D, n);
    return hipGetLastError() == hipSuccess ? GSS_OK : GSS_EHIP;
  }
  if (!small) return run_wpe_large(ctx, Yc, T_len, S, F, Tmax, D, taps, delay, iters, Xc, st);
  switch (D) {
#define GSS_CASE_D(DD) \
  case DD: return run_wpe<DD>(ctx, Yc, T_len, S, F, Tmax, taps, delay, iters, Xc, st);
    GSS_CASE_D(1) GSS_CASE_D(2) GSS_CASE_D(3) GSS_CASE_D(4) GSS_CASE_D(5) GSS_CASE_D(6) GSS_CASE_D(7) GSS_CASE_D(8)
#undef GSS_CASE_D
    default: return GSS_EUNSUPPORTED;
  }
}
