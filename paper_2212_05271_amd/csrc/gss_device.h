// Device-side building blocks shared by the EM and the MVDR kernels (internal, not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <type_traits>

#include "gss_internal.h"

namespace {

constexpr int kWave = 64;

__host__ __device__ constexpr int next_pow2(int x) {
  int p = 1;
  while (p < x) p <<= 1;
  return p;
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

// One Newton step only: relative error about 2e-15 (the hardware estimate is good to 5e-8).  For the
// posterior's 1 / q and 1 / Z, where a few ulps change nothing that survives the fp32 output.
__device__ __forceinline__ double rcp_f64_fast(double x) {
  const double r = __builtin_amdgcn_rcp(x);
  return fma(fma(-x, r, 1.0), r, r);
}

// Sum of a double over the 64 lanes of the wavefront, the same value in every lane, in a fixed order.  Within
// a row of 16 lanes four butterfly steps through the lane-permute modifier of the vector move (on the two
// halves of the double): neighbours, pairs, the mirrored half of 8, the mirrored row; then the four row sums
// are read into scalar registers and added.  No LDS traffic (a shuffle goes through the LDS crossbar and costs
// a round trip per step).
__device__ __forceinline__ double wave_sum_f64(double v) {
  auto step = [](double x, auto CTRL) {
    constexpr int ctrl = decltype(CTRL)::value;
    const int lo = __double2loint(x), hi = __double2hiint(x);
    const int plo = __builtin_amdgcn_update_dpp(0, lo, ctrl, 0xf, 0xf, false);
    const int phi = __builtin_amdgcn_update_dpp(0, hi, ctrl, 0xf, 0xf, false);
    return x + __hiloint2double(phi, plo);
  };
  v = step(v, std::integral_constant<int, 0xB1>{});     // quad_perm [1, 0, 3, 2]
  v = step(v, std::integral_constant<int, 0x4E>{});     // quad_perm [2, 3, 0, 1]
  v = step(v, std::integral_constant<int, 0x141>{});    // row_half_mirror
  v = step(v, std::integral_constant<int, 0x140>{});    // row_mirror
  const int lo = __double2loint(v), hi = __double2hiint(v);
  double r[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
    r[q] = __hiloint2double(__builtin_amdgcn_readlane(hi, 16 * q), __builtin_amdgcn_readlane(lo, 16 * q));
  return (r[0] + r[1]) + (r[2] + r[3]);
}

// The value that lane 8 * (lane / 8) + N holds, in every lane of that group of 8: a row of 16 lanes is served by
// two lane-permute moves, each confined to one half of the row by its bank mask.  Every lane of the wavefront
// must be active.  (s_nop: a vector write of the source needs two wait states before the permute reads it.)
template <int N>
__device__ __forceinline__ double class_row_bcast(double src) {
  double r;
  asm("s_nop 1\n\tv_mov_b64_dpp %0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0x3\n\t"
      "v_mov_b64_dpp %0, %1 row_newbcast:%3 row_mask:0xf bank_mask:0xc"
      : "=&v"(r)
      : "v"(src), "n"(N), "n"(N + 8));
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

// Sums of N per-lane doubles over the 64 lanes of the wavefront, all at once and in a fixed order: six
// butterfly steps, and at each step a lane keeps only half of its values (of each pair of values one lane of
// the exchanging pair keeps the first and the other the second), so the work halves from step to step
// instead of every value paying six steps.  Afterwards lane l holds in v[j] the wavefront's total of value
// 64 j + transposed_index(l) (where that is below N; the other entries are meaningless).  The first four steps
// stay inside a row of 16 lanes and use the lane-permute modifier of the vector move (mirrored row, mirrored
// half, pairs, neighbours, in this order: each permutation leaves the bits that earlier steps selected on
// unchanged), the last two cross the rows with a shuffle.  Every lane of the wavefront must be active.
template <int CTRL>
__device__ __forceinline__ double dpp_permute_f64(double x) {
  const int lo = __double2loint(x), hi = __double2hiint(x);
  const int plo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xf, 0xf, false);
  const int phi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xf, 0xf, false);
  return __hiloint2double(phi, plo);
}
__device__ __forceinline__ int transposed_index(int lane) {
  return (int)(__brev((unsigned)(lane & 15)) >> 28) | (lane & 48);
}
// ROWS_ONLY: only the four steps inside the rows of 16 lanes: lane l then holds in v[j] the sum over its row of
// value 16 j + transposed_index(l & 15), and the caller adds the four rows itself.
template <int N, bool ROWS_ONLY = false>
__device__ __forceinline__ void transpose_reduce(double (&v)[N], int lane) {
  auto step = [&](auto CNT, bool second, auto perm) {
    constexpr int n = decltype(CNT)::value;
    static_for<0, n / 2>([&](auto MI) {
      constexpr int m = MI.value;
      const double a = v[2 * m], b = v[2 * m + 1];
      const double keep = second ? b : a, send = second ? a : b;
      v[m] = keep + perm(send);
    });
    if constexpr (n & 1) {            // a value without a partner: both lanes keep its sum
      const double a = v[n - 1];
      v[n / 2] = a + perm(a);
    }
  };
  constexpr int n1 = (N + 1) / 2, n2 = (n1 + 1) / 2, n3 = (n2 + 1) / 2, n4 = (n3 + 1) / 2, n5 = (n4 + 1) / 2;
  step(std::integral_constant<int, N>{}, (lane & 8) != 0, [](double x) { return dpp_permute_f64<0x140>(x); });   // row_mirror
  step(std::integral_constant<int, n1>{}, (lane & 4) != 0, [](double x) { return dpp_permute_f64<0x141>(x); });  // row_half_mirror
  step(std::integral_constant<int, n2>{}, (lane & 2) != 0, [](double x) { return dpp_permute_f64<0x4E>(x); });   // quad_perm [2, 3, 0, 1]
  step(std::integral_constant<int, n3>{}, (lane & 1) != 0, [](double x) { return dpp_permute_f64<0xB1>(x); });   // quad_perm [1, 0, 3, 2]
  if constexpr (!ROWS_ONLY) {
    step(std::integral_constant<int, n4>{}, (lane & 16) != 0, [](double x) { return __shfl_xor(x, 16, kWave); });
    step(std::integral_constant<int, n5>{}, (lane & 32) != 0, [](double x) { return __shfl_xor(x, 32, kWave); });
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

// First frame of (segment s, frequency f) in the view and the number T of valid frames of the segment:
// T_len[s] (all Tmax frames if T_len is NULL) clipped to [0, Tmax] and to what the underlying array holds
// behind the segment's first frame.
__device__ __forceinline__ const float2* y_row(const gss_yview& v, const int32_t* __restrict__ T_len, int s, int f,
                                               int D, int Tmax, int& T) {
  long off = v.frame0 ? (long)v.frame0[s] : 0;
  off = off < 0 ? 0 : (off > v.t_limit ? v.t_limit : off);
  int t = T_len ? T_len[s] : Tmax;
  t = t < 0 ? 0 : (t > Tmax ? Tmax : t);
  const long room = v.t_limit - off;
  T = (long)t > room ? (int)room : t;
  return v.base + (long)s * v.s_stride + (long)f * v.f_stride + off * D;
}
__device__ __forceinline__ int y_frames(const gss_yview& v, const int32_t* __restrict__ T_len, int s, int Tmax) {
  int T;
  (void)y_row(v, T_len, s, 0, 1, Tmax, T);
  return T;
}

// Orders this wavefront's LDS traffic: everything written before is visible to every lane of the
// wavefront after.  (The LDS executes one wavefront's instructions in order; this only has to stop the
// compiler from moving accesses across and make it wait for outstanding ones.)
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A class whose bit is clear in a tile's activity mask has posterior 0 in every frame of the tile and adds nothing
// to any sum: the pass kernels skip its arithmetic for the whole tile under wave-uniform branches.
// Activity in the form the pass kernels read: abyte[s][t] has bit k set when class k may be active in frame t
// (a_{t,k} of Eq. (5); 0 at t >= T_len[s]), tmask[s][tile] is the OR of the bytes of the tile's 64 frames.
// Grid: one wavefront per (segment, tile).
__global__ __launch_bounds__(kWave) void em_pack_activity(
    gss_yview yv, const uint8_t* __restrict__ act, const int32_t* __restrict__ T_len, uint8_t* __restrict__ abyte,
    uint32_t* __restrict__ tmask, int K, int Tmax, int tiles) {
  const int s = blockIdx.x / tiles, tile = blockIdx.x % tiles;
  const int lane = threadIdx.x;
  const int T = y_frames(yv, T_len, s, Tmax);
  const int t = tile * kWave + lane;
  unsigned b = 0;
  if (t < T)
    for (int k = 0; k < K; ++k) b |= (act[((long)s * K + k) * Tmax + t] != 0 ? 1u : 0u) << k;
  if (t < Tmax) abyte[(long)s * Tmax + t] = (uint8_t)b;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) b |= (unsigned)__shfl_xor((int)b, off, kWave);
  if (lane == 0) tmask[(long)s * tiles + tile] = b;
}

// acc += c[lane N of the row] * p: the double-precision FMA with the row-broadcast selector on its first
// factor.  Every lane of the wavefront must be active (the selector reads other lanes).  The instruction is
// written as an asm statement, which hides it from the compiler's hazard handling: a lane-selecting
// instruction must not issue within two wait states of a vector instruction that writes one of its
// registers, so the first FMA of a run (SETTLE) is preceded by the two idle states itself.
template <int N, bool SETTLE>
__device__ __forceinline__ void fma_bcast(double& acc, double c, double p) {
  static_assert(N >= 0 && N < 16, "row_newbcast selects one of the 16 lanes of a row");
  if constexpr (SETTLE)
    asm("s_nop 1\n\tv_fmac_f64_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
        : "+v"(acc) : "v"(c), "v"(p), "n"(N));
  else
    asm("v_fmac_f64_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(c), "v"(p), "n"(N));
}

// q0 += sum over u < n of c[2 u] re[u] and q1 += sum over u < n of c[2 u + 1] im[u], 1 <= n (8 and more: all 8
// items), c[x] being the value that `c` holds in lane x of the lane's row of 16.  n must be the same in every lane.
// The items run from the last to the first, and a shorter run enters the chain further down, so each accumulator
// stays in one register whatever n is (a switch over n in C++ gives every length its own copy of the chain and
// moves the accumulators between the copies' registers around every one of them).  Idle states: the two scalar
// instructions in front of every entry separate the first FMA from the last vector write before the statement,
// and within the chain an accumulator is read two issue slots after it was written, one of them the s_nop.
__device__ __forceinline__ void fma_bcast_run(double& q0, double& q1, double c, const double (&re)[8],
                                              const double (&im)[8], int n) {
#define GSS_BCAST_ITEM(label, u, a, b)                                                               \
  label ":\n\t"                                                                                      \
  "v_fmac_f64_dpp %[q0], %[c], %[re" #u "] row_newbcast:" #a " row_mask:0xf bank_mask:0xf\n\t"        \
  "v_fmac_f64_dpp %[q1], %[c], %[im" #u "] row_newbcast:" #b " row_mask:0xf bank_mask:0xf\n\t"
  asm("s_cmp_gt_i32 %[n], 7\n\t"
      "s_cbranch_scc1 18f\n\t"
      "s_cmp_gt_i32 %[n], 3\n\t"
      "s_cbranch_scc1 10f\n\t"
      "s_cmp_eq_u32 %[n], 3\n\t"
      "s_cbranch_scc1 13f\n\t"
      "s_cmp_eq_u32 %[n], 2\n\t"
      "s_cbranch_scc1 12f\n\t"
      "s_branch 11f\n\t"
      "10:\n\t"
      "s_cmp_eq_u32 %[n], 7\n\t"
      "s_cbranch_scc1 17f\n\t"
      "s_cmp_eq_u32 %[n], 6\n\t"
      "s_cbranch_scc1 16f\n\t"
      "s_cmp_eq_u32 %[n], 5\n\t"
      "s_cbranch_scc1 15f\n\t"
      "s_branch 14f\n\t"
      GSS_BCAST_ITEM("18", 7, 14, 15) "s_nop 0\n\t"
      GSS_BCAST_ITEM("17", 6, 12, 13) "s_nop 0\n\t"
      GSS_BCAST_ITEM("16", 5, 10, 11) "s_nop 0\n\t"
      GSS_BCAST_ITEM("15", 4, 8, 9) "s_nop 0\n\t"
      GSS_BCAST_ITEM("14", 3, 6, 7) "s_nop 0\n\t"
      GSS_BCAST_ITEM("13", 2, 4, 5) "s_nop 0\n\t"
      GSS_BCAST_ITEM("12", 1, 2, 3) "s_nop 0\n\t"
      GSS_BCAST_ITEM("11", 0, 0, 1)
      : [q0] "+v"(q0), [q1] "+v"(q1)
      : [c] "v"(c), [n] "s"(n), [re0] "v"(re[0]), [re1] "v"(re[1]), [re2] "v"(re[2]), [re3] "v"(re[3]),
        [re4] "v"(re[4]), [re5] "v"(re[5]), [re6] "v"(re[6]), [re7] "v"(re[7]), [im0] "v"(im[0]), [im1] "v"(im[1]),
        [im2] "v"(im[2]), [im3] "v"(im[3]), [im4] "v"(im[4]), [im5] "v"(im[5]), [im6] "v"(im[6]), [im7] "v"(im[7])
      : "scc");
#undef GSS_BCAST_ITEM
}

// Wave-uniform test of bit k of `mask`, re-evaluated from the one scalar register that holds the mask at every
// use (the empty asm statement keeps the compiler from caching the K booleans in scalar register pairs).
__device__ __forceinline__ bool class_on(unsigned mask, int k) {
  asm volatile("" : "+s"(mask));
  return (mask >> k) & 1u;
}

// Tile geometry shared by the kernels that accumulate weighted outer products: a workgroup is
// kPassWaves wavefronts, each wavefront owns whole tiles of 64 frames and a private LDS region.
constexpr int kPassWaves = 4;
// Doubles per frame row of the y tile: the 8 complex channels, then -i y_c for the channels c < 4 (the lanes that
// pair a channel with the one four below it read that copy, see slot_entry), then 2 of padding (16-byte units: 13
// per row, odd, so that the rows of adjacent frames start in different banks).
constexpr int kYStride = 26;
constexpr int kYTurned = 16;   // offset of the turned copies within a row
static_assert(kYStride == kYTurned + 8 + 2, "a row is 8 channels, 4 turned copies and two padding entries");

// Writes one frame row of the y tile: channel d at 2 d (zero beyond D) and the turned copies of channels 0..3.
template <int D>
__device__ __forceinline__ void store_tile_row(double* __restrict__ row, const double (&yr)[D], const double (&yi)[D]) {
#pragma unroll
  for (int d = 0; d < 8; ++d) {
    double2 yv = make_double2(0.0, 0.0);
    if (d < D) yv = make_double2(yr[d < D ? d : 0], yi[d < D ? d : 0]);
    *reinterpret_cast<double2*>(&row[2 * d]) = yv;
    if (d < 4) *reinterpret_cast<double2*>(&row[kYTurned + 2 * d]) = make_double2(yv.y, -yv.x);
  }
}


// Phase-2 lane type eg = channel i.  Its 8 accumulator slots: n = 0..5 are Re and Im of y_i conj(y_b),
// b = (i + d) mod 8 for d = 1, 2, 3; n = 6 is the real diagonal entry |y_i|^2; n = 7 is one half of the pair at
// distance 4: Re of y_i conj(y_(i+4)) for i < 4 and Im of y_(i-4) conj(y_i) for i >= 4.  Both halves are
// y_i.re * a + y_i.im * b of a second operand (a, b) = y_(i+4) or -i y_(i-4), which the lane reads from the tile
// (the row holds the turned copies), so every lane type runs the same instructions.  The pairs at circular
// distance 1..4 are all 28 pairs once; where b < i the slot holds the conjugate of the stored (upper-triangle)
// entry, i.e. its imaginary part with the opposite sign.
struct SlotEntry { int i, j, part, sign; };     // part: 0 real diagonal, 1 Re, 2 Im
__host__ __device__ constexpr SlotEntry slot_entry(int eg, int n) {
  if (n < 6) {
    const int d = n / 2 + 1;
    const int part = 1 + (n & 1);
    const int a = eg, b = (eg + d) % 8;
    if (a < b) return SlotEntry{a, b, part, 1};
    return SlotEntry{b, a, part, part == 2 ? -1 : 1};
  }
  if (n == 6) return SlotEntry{eg, eg, 0, 1};
  return eg < 4 ? SlotEntry{eg, eg + 4, 1, 1} : SlotEntry{eg - 4, eg, 2, 1};
}

// Packed index (gss_packed_row order, matrix size D) of accumulator slot n of lane type eg, or -1 if the
// slot lies in the zero padding.
__host__ __device__ constexpr int slot_packed_index(int eg, int n, int D) {
  const SlotEntry e = slot_entry(eg, n);
  if (e.i >= D || e.j >= D) return -1;
  return e.part == 0 ? gss_packed_row(e.i, D) : gss_packed_row(e.i, D) + 1 + 2 * (e.j - e.i - 1) + (e.part - 1);
}

// slot_packed_index for every matrix size 1..8 and slot eg * 8 + n, and the slot's sign, as tables.
struct SlotTable { short v[9][64]; signed char sign[64]; };
constexpr SlotTable make_slot_table() {
  SlotTable t{};
  for (int d = 0; d <= 8; ++d)
    for (int sl = 0; sl < 64; ++sl) t.v[d][sl] = d == 0 ? (short)-1 : (short)slot_packed_index(sl / 8, sl % 8, d);
  for (int sl = 0; sl < 64; ++sl) t.sign[sl] = (signed char)slot_entry(sl / 8, sl % 8).sign;
  return t;
}

// Phase 2 of a tile: lane (tg, eg) accumulates acc[n][k] += w_k[r] * (slot n of lane type eg)[r] over its 8
// frames r = tg, tg + 8, ... of the 64-frame tile in LDS.  sY: [64][kYStride] doubles (8 complex channels
// per frame, zero beyond D), sW: [64][WS] doubles (KW weights per frame).
template <int KW, int WS, int UNROLL = 2>
__device__ __forceinline__ void accumulate_tile(const double* __restrict__ sY, const double* __restrict__ sW,
                                                int tg, int eg, double (&acc)[8][KW]) {
  const int c1 = 2 * ((eg + 1) & 7), c2 = 2 * ((eg + 2) & 7), c3 = 2 * ((eg + 3) & 7);
  const int c4 = eg < 4 ? 2 * (eg + 4) : kYTurned + 2 * (eg - 4);
#pragma unroll UNROLL
  for (int j = 0; j < 8; ++j) {
    const int r = tg + 8 * j;              // rows of the 8 frame groups are adjacent: distinct LDS banks
    double w[KW];
#pragma unroll
    for (int k = 0; k < KW; ++k) w[k] = sW[r * WS + k];
    const double* __restrict__ row = sY + r * kYStride;
    const double2 x = *reinterpret_cast<const double2*>(&row[2 * eg]);
    const double2 y1 = *reinterpret_cast<const double2*>(&row[c1]);
    const double2 y2 = *reinterpret_cast<const double2*>(&row[c2]);
    const double2 y3 = *reinterpret_cast<const double2*>(&row[c3]);
    const double2 y4 = *reinterpret_cast<const double2*>(&row[c4]);
    double e[8];
    e[0] = x.x * y1.x + x.y * y1.y;  e[1] = x.y * y1.x - x.x * y1.y;
    e[2] = x.x * y2.x + x.y * y2.y;  e[3] = x.y * y2.x - x.x * y2.y;
    e[4] = x.x * y3.x + x.y * y3.y;  e[5] = x.y * y3.x - x.x * y3.y;
    e[6] = x.x * x.x + x.y * x.y;    e[7] = x.x * y4.x + x.y * y4.y;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
#pragma unroll
      for (int k = 0; k < KW; ++k) acc[n][k] = fma(w[k], e[n], acc[n][k]);
    }
  }
}

// The same for the classes of `mask` only (wave-uniform): the weights of the other classes are zero in every
// frame of the tile (their columns of sW hold stale values that are read and never used).  One frame per
// step: its entries are formed, the row and weights of the next frame are requested from LDS, and then each
// class of the mask adds its 8 products under one uniform branch, so the LDS latency is covered by the
// previous frame's arithmetic.
template <int KW, int WS>
__device__ __forceinline__ void accumulate_tile_masked(const double* __restrict__ sY, const double* __restrict__ sW,
                                                       int tg, int eg, unsigned mask, double (&acc)[8][KW]) {
  // five row pointers and one weight pointer per lane; every access below is one of them plus a constant
  // (the constant goes into the offset field of the LDS instruction)
  const double* __restrict__ p0 = sY + tg * kYStride + 2 * eg;
  const double* __restrict__ p1 = sY + tg * kYStride + 2 * ((eg + 1) & 7);
  const double* __restrict__ p2 = sY + tg * kYStride + 2 * ((eg + 2) & 7);
  const double* __restrict__ p3 = sY + tg * kYStride + 2 * ((eg + 3) & 7);
  const double* __restrict__ p4 = sY + tg * kYStride + (eg < 4 ? 2 * (eg + 4) : kYTurned + 2 * (eg - 4));
  const double* __restrict__ pw = sW + tg * WS;
  double2 y[5];
  double w[KW];
  auto fetch = [&](auto JF) {
    constexpr int o = 8 * JF.value * kYStride;     // rows of the 8 frame groups are adjacent: distinct LDS banks
    y[0] = *reinterpret_cast<const double2*>(p0 + o);
    y[1] = *reinterpret_cast<const double2*>(p1 + o);
    y[2] = *reinterpret_cast<const double2*>(p2 + o);
    y[3] = *reinterpret_cast<const double2*>(p3 + o);
    y[4] = *reinterpret_cast<const double2*>(p4 + o);
#pragma unroll
    for (int k = 0; k < KW; ++k) w[k] = pw[8 * JF.value * WS + k];
  };
  fetch(std::integral_constant<int, 0>{});
  static_for<0, 8>([&](auto JI) {
    constexpr int j = JI.value;
    double e[8], wc[KW];
    {
      const double2 x = y[0], y1 = y[1], y2 = y[2], y3 = y[3], y4 = y[4];
      e[0] = x.x * y1.x + x.y * y1.y;  e[1] = x.y * y1.x - x.x * y1.y;
      e[2] = x.x * y2.x + x.y * y2.y;  e[3] = x.y * y2.x - x.x * y2.y;
      e[4] = x.x * y3.x + x.y * y3.y;  e[5] = x.y * y3.x - x.x * y3.y;
      e[6] = x.x * x.x + x.y * x.y;    e[7] = x.x * y4.x + x.y * y4.y;
#pragma unroll
      for (int k = 0; k < KW; ++k) wc[k] = w[k];
    }
    if constexpr (j < 7) fetch(std::integral_constant<int, j + 1>{});
    static_for<0, KW>([&](auto KI) {
      constexpr int k = KI.value;
      unsigned m = mask;
      asm volatile("" : "+s"(m));           // re-test the one mask register instead of keeping KW booleans
      if ((m >> k) & 1u) {
#pragma unroll
        for (int n = 0; n < 8; ++n) acc[n][k] = fma(wc[k], e[n], acc[n][k]);
      }
    });
  });
}

// Reduction of the per-lane accumulators of a workgroup of kPassWaves wavefronts into packed partial
// sums: out[k * E + packed index] for k < KW, matrix size D.  Sums are taken in a fixed order (frame
// groups ascending, then wavefronts ascending).
//   wbuf: LDS private to the calling wavefront, kReduceWaveDoubles doubles (its tile region);
//   red:  LDS scratch of the workgroup, kPassWaves * (64 * KW + KW) doubles, may overlap the wbuf regions.
// WITH_N: nvals[k] is one more per-lane partial sum per class (lane = frame layout), summed over all lanes and
// wavefronts into nout[k].
// The function starts with a barrier (every wavefront is done with its tiles).  First every wavefront
// sums over its 8 frame groups through its own LDS region, two classes at a time: entry n of all lanes
// goes out as one contiguous row (lane = 8 tg + eg), and lane o = 8 n + eg reads the 8 values of slot
// (eg, n) back.  Then the wavefronts' sums meet in `red`.
constexpr int kReduceRow = 72;                         // doubles per row of 64 (+ 8: spreads the banks)
constexpr int kReduceWaveDoubles = 2 * 8 * kReduceRow;
static_assert(kReduceWaveDoubles <= kWave * kYStride, "the y tile of a wavefront must hold its reduction rows");

template <int D, int KW, bool WITH_N>
__device__ __forceinline__ void reduce_and_store_partials(double (&acc)[8][KW], double (&nvals)[KW], double* wbuf,
                                                          double* red, double* __restrict__ out,
                                                          double* __restrict__ nout, int lane, int wave) {
  constexpr int E = D * D;
  double S[KW];
  if constexpr (WITH_N) {                    // per-lane scalars (one per class): summed over the wavefront
#pragma unroll
    for (int k = 0; k < KW; ++k) {
      double nv = wave_sum_f64(nvals[k]);
      nvals[k] = nv;
    }
  }
  __syncthreads();
#pragma unroll
  for (int k0 = 0; k0 < KW; k0 += 2) {
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      if (k0 + c < KW) {
#pragma unroll
        for (int n = 0; n < 8; ++n) wbuf[(c * 8 + n) * kReduceRow + lane] = acc[n][k0 + c];
      }
    }
    wave_lds_sync();
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      if (k0 + c < KW) {
        double sum = 0.0;
#pragma unroll
        for (int tg = 0; tg < 8; ++tg) sum += wbuf[(c * 8 + (lane >> 3)) * kReduceRow + tg * 8 + (lane & 7)];
        S[k0 + c] = sum;
      }
    }
    wave_lds_sync();
  }
  __syncthreads();                           // the private regions are free: `red` may overlap them
  double* redn = red + kPassWaves * 64 * KW;
#pragma unroll
  for (int k = 0; k < KW; ++k) red[(wave * KW + k) * 64 + (lane & 7) * 8 + (lane >> 3)] = S[k];
  if constexpr (WITH_N) {
    if (lane == 0) {
#pragma unroll
      for (int k = 0; k < KW; ++k) redn[wave * KW + k] = nvals[k];
    }
  }
  __syncthreads();
  for (int x = threadIdx.x; x < 64 * KW; x += kWave * kPassWaves) {
    const int k = x / 64, slot = x % 64;
    double sum = 0.0;
#pragma unroll
    for (int w = 0; w < kPassWaves; ++w) sum += red[(w * KW + k) * 64 + slot];
    static constexpr SlotTable kSlotTable = make_slot_table();
    const int pidx = kSlotTable.v[D][slot];   // slot -> packed index for matrix size D; padding slots are dropped
    if (pidx >= 0) out[k * E + pidx] = kSlotTable.sign[slot] < 0 ? -sum : sum;
  }
  if constexpr (WITH_N) {
    if (threadIdx.x < KW) {
      double sum = 0.0;
#pragma unroll
      for (int w = 0; w < kPassWaves; ++w) sum += redn[w * KW + threadIdx.x];
      nout[threadIdx.x] = sum;
    }
  }
}

// Workgroups of `threads` threads of kernel `kern` that one compute unit holds at a time (`dflt` if the
// runtime cannot say).
template <typename Kern>
inline int resident_wgs(Kern kern, int threads, int dflt, size_t lds_bytes = 0) {
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, threads, lds_bytes) != hipSuccess || n < 1) {
    (void)hipGetLastError();
    n = dflt;
  }
  return n;
}

// How the (segment, frequency) problems are cut into workgroups.  The first n_main problems get c_main
// chunks of tpc_main tiles each; the remaining ones (the tail that would otherwise run alone on an almost
// empty chip after the last full round of workgroups) are cut finer, into c_tail chunks of tpc_tail tiles.
// Workgroup b writes partial-sum slot b.
struct ChunkMap {
  int n_main, c_main, tpc_main, c_tail, tpc_tail;
};
__host__ __device__ inline void chunk_decode(const ChunkMap& m, unsigned b, long& sf, int& chunk, int& tpc) {
  // 32-bit arithmetic: the grid has fewer than 2^31 workgroups
  const unsigned main_wgs = (unsigned)m.n_main * (unsigned)m.c_main;
  if (b < main_wgs) {
    sf = (long)(b / (unsigned)m.c_main);
    chunk = (int)(b % (unsigned)m.c_main);
    tpc = m.tpc_main;
  } else {
    const unsigned r = b - main_wgs;
    sf = (long)((unsigned)m.n_main + r / (unsigned)m.c_tail);
    chunk = (int)(r % (unsigned)m.c_tail);
    tpc = m.tpc_tail;
  }
}
__host__ __device__ inline long chunk_base(const ChunkMap& m, long sf, int& count) {
  if (sf < m.n_main) {
    count = m.c_main;
    return sf * m.c_main;
  }
  count = m.c_tail;
  return (long)m.n_main * m.c_main + (sf - m.n_main) * m.c_tail;
}

inline long chunk_map_wgs(const ChunkMap& m, long n_sf) {
  return (long)m.n_main * m.c_main + (n_sf - m.n_main) * m.c_tail;
}

// Chunking of n_sf problems of `tiles` tiles each for a kernel with `slots` resident workgroups; chunks are
// multiples of `round_up` tiles.  Splitting a problem over several workgroups costs a partial-sum round
// trip and a second reduction, so it is done only as far as needed to fill the slots (tpc_override > 0
// fixes the tiles per chunk of the main part instead).  Tail: if the workgroups left over after the last
// full round of slots fill less than a quarter of the chip, the problems they belong to are cut finer so
// that the remainder spreads out.
inline ChunkMap plan_chunk_map(long slots, long n_sf, int tiles, int round_up, int tpc_override, bool allow_tail) {
  ChunkMap m;
  auto chunks_for = [&](int tpc) { return (tiles + tpc - 1) / tpc; };
  auto tpc_for = [&](long c) {
    int tpc = (int)((tiles + c - 1) / c);
    tpc = (tpc + round_up - 1) / round_up * round_up;
    return tpc;
  };
  long c_target = (slots + n_sf - 1) / n_sf;
  if (c_target < 1) c_target = 1;
  m.tpc_main = tpc_override > 0 ? tpc_override : tpc_for(c_target);
  m.c_main = chunks_for(m.tpc_main);
  m.n_main = (int)n_sf;
  m.c_tail = m.c_main;
  m.tpc_tail = m.tpc_main;
  const long wgs = n_sf * m.c_main;
  const long rem = wgs % slots;
  if (allow_tail && wgs > slots && rem > 0 && rem * 4 <= slots) {
    const long tail_sf = (rem + m.c_main - 1) / m.c_main;
    const long want = slots / (2 * tail_sf) > 1 ? slots / (2 * tail_sf) : 1;    // chunks per tail problem
    const int tpc_t = tpc_for(want * m.c_main);
    if (tpc_t < m.tpc_main) {
      m.n_main = (int)(n_sf - tail_sf);
      m.tpc_tail = tpc_t;
      m.c_tail = chunks_for(tpc_t);
    }
  }
  return m;
}


}  // namespace
