// Column-mode passes: the stages of a processor applied along the ROW index of a row-major
// matrix, M <- U^T M (or U M), without transposing it (two-sided weight rotation W~ = U^T W V,
// Sec. 2; stage arithmetic of Algorithm 1 with the matrix row as the coordinate).
//
// Stage t couples rows i = alpha b s + r s + beta, r < b, of EVERY column with the same block
// K_t[alpha s + beta], so along a row the work is perfectly coalesced and a block's b*b values
// are uniform over a wave: the blocks a tile needs (at most 9 KB) travel with it, requested
// together with its rows and read from LDS as broadcasts.  A pass is a run of consecutive
// stages whose radices multiply to P <= 128; a workgroup owns a tile of P rows (row0 + j S,
// j < P, S = the run's lowest stride) x 128 columns in LDS as float32 (two columns per lane),
// executes the run's stages on it (one barrier per step; up to three consecutive radix-2
// stages share one LDS round trip, eight rows in registers) and writes it back.  Tiles are
// disjoint, so a pass may run in place.  2^13 rows take two passes (7 + 6 stages): the matrix
// moves through device memory twice instead of the five times of transpose / row kernels /
// transpose.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <type_traits>

#include "harp_internal.h"

namespace harp {
namespace {

constexpr int kColCols = 128;      // columns per tile
constexpr int kColThreads = 256;   // 4 waves
constexpr int kColWaves = kColThreads / 64;
constexpr int kColMaxP = 128;      // rows per tile (LDS: P * 128 * 4 bytes = 64 KB)
constexpr int kColParPerThread = 9;
constexpr int kColMaxPar = kColParPerThread * kColThreads;   // block values per tile (9 KB)

__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {   // round to nearest even
  // branch-free: a branch between the stores would hide their number from the compiler's
  // count of outstanding memory operations
  const uint32_t u = __float_as_uint(f);
  const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  const uint32_t quiet = (u >> 16) | 0x40u;
  return ((u & 0x7fffffffu) > 0x7f800000u) ? quiet : rounded;
}

// Two adjacent elements as loaded (no arithmetic on them until they are needed, so that the
// loads of the next tile stay in flight during the work on the current one).
// zh16 = block-scaled halves (the workspace of bf16 callers): the pair's two halves plus the
// exponent byte of its 16-column segment, which lies `eoff` bytes behind the pair (eight lanes
// share a segment and read the same byte).  Other element types ignore eoff.
template <typename T> struct ColRaw;
template <> struct ColRaw<float> { float2 v; };
template <> struct ColRaw<uint16_t> { uint32_t lo, hi; };   // VEC: both in lo
template <> struct ColRaw<zh16> { uint32_t h, e; };

template <typename T, bool VEC>
__device__ __forceinline__ void col_load(ColRaw<T> &r, const T *p, bool v0, bool v1, int eoff);
template <>
__device__ __forceinline__ void col_load<float, true>(ColRaw<float> &r, const float *p, bool v0, bool, int) {
  r.v = v0 ? *reinterpret_cast<const float2 *>(p) : make_float2(0.f, 0.f);
}
template <>
__device__ __forceinline__ void col_load<float, false>(ColRaw<float> &r, const float *p, bool v0, bool v1, int) {
  r.v = make_float2(v0 ? p[0] : 0.f, v1 ? p[1] : 0.f);
}
template <>
__device__ __forceinline__ void col_load<uint16_t, true>(ColRaw<uint16_t> &r, const uint16_t *p, bool v0, bool, int) {
  r.lo = v0 ? *reinterpret_cast<const uint32_t *>(p) : 0u;
  r.hi = 0u;
}
template <>
__device__ __forceinline__ void col_load<uint16_t, false>(ColRaw<uint16_t> &r, const uint16_t *p, bool v0, bool v1, int) {
  r.lo = v0 ? (uint32_t)p[0] : 0u;
  r.hi = v1 ? (uint32_t)p[1] : 0u;
}
template <>
__device__ __forceinline__ void col_load<zh16, true>(ColRaw<zh16> &r, const zh16 *p, bool, bool, int eoff) {
  r.h = *reinterpret_cast<const uint32_t *>(p);
  r.e = reinterpret_cast<const uint8_t *>(p)[eoff];
}
template <bool VEC>
__device__ __forceinline__ float2 col_widen(const ColRaw<float> &r) { return r.v; }
template <bool VEC>
__device__ __forceinline__ float2 col_widen(const ColRaw<uint16_t> &r) {
  if (VEC) return make_float2(__uint_as_float(r.lo << 16), __uint_as_float(r.lo & 0xffff0000u));
  return make_float2(__uint_as_float(r.lo << 16), __uint_as_float(r.hi << 16));
}
template <bool VEC>
__device__ __forceinline__ float2 col_widen(const ColRaw<zh16> &r) {
  float2 v;
  z16_unpack(r.h, z16_up(r.e), v.x, v.y);
  return v;
}

template <typename T, bool VEC>
__device__ __forceinline__ void col_store(T *p, float2 v, bool v0, bool v1, int eoff);
template <>
__device__ __forceinline__ void col_store<float, true>(float *p, float2 v, bool v0, bool, int) {
  if (v0) *reinterpret_cast<float2 *>(p) = v;
}
template <>
__device__ __forceinline__ void col_store<float, false>(float *p, float2 v, bool v0, bool v1, int) {
  if (v0) p[0] = v.x;
  if (v1) p[1] = v.y;
}
template <>
__device__ __forceinline__ void col_store<uint16_t, true>(uint16_t *p, float2 v, bool v0, bool, int) {
  if (v0) *reinterpret_cast<uint32_t *>(p) = f32_to_bf16(v.x) | (f32_to_bf16(v.y) << 16);
}
template <>
__device__ __forceinline__ void col_store<uint16_t, false>(uint16_t *p, float2 v, bool v0, bool v1, int) {
  if (v0) p[0] = (uint16_t)f32_to_bf16(v.x);
  if (v1) p[1] = (uint16_t)f32_to_bf16(v.y);
}
// The eight lanes of a segment find its largest magnitude with three DPP steps (bit patterns of
// non-negative floats order like unsigned integers); every one of them writes the exponent byte
// (same address, same value), so that no store is conditional.  Unguarded tiles only: every lane
// of an aligned group of eight holds a pair of the same segment.
template <>
__device__ __forceinline__ void col_store<zh16, true>(zh16 *p, float2 v, bool, bool, int eoff) {
  uint32_t mx = __float_as_uint(fmaxf(fabsf(v.x), fabsf(v.y)));
  mx = max(mx, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mx, 0xB1 /* quad_perm [1,0,3,2] */, 0xf, 0xf, false));
  mx = max(mx, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mx, 0x4E /* quad_perm [2,3,0,1] */, 0xf, 0xf, false));
  mx = max(mx, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mx, 0x141 /* row_half_mirror */, 0xf, 0xf, false));
  uint32_t ex = mx >> 23;
  ex = ex > 253u ? 253u : ex;
  const float f = z16_down(ex);
  *reinterpret_cast<uint32_t *>(p) = z16_pack(v.x * f, v.y * f);
  reinterpret_cast<uint8_t *>(p)[eoff] = (uint8_t)ex;
}
template <typename T> struct IsZ16 { static constexpr bool value = false; };
template <> struct IsZ16<zh16> { static constexpr bool value = true; };

// Workgroup id -> logical id such that G logically consecutive workgroups (neighbouring column
// positions of the same rows: they share 128-byte lines -- of exponent bytes, and of data where a
// tile row is shorter than a line) run on one XCD next to each other in dispatch order, so the
// line is fetched from device memory once, into that XCD's L2 (workgroup b runs on XCD b mod 8).
// The grid is a multiple of 8 G (checked by the launcher); G == 0: identity.
__device__ __forceinline__ unsigned xcd_grouped(unsigned b, unsigned G) {
  if (G == 0) return b;
  const unsigned xcd = b & 7u, k = b >> 3;
  return ((k / G) * 8u + xcd) * G + (k % G);
}
inline unsigned xcd_group_size(int64_t positions, int64_t grid, int cap) {
  for (int g = cap; g >= 2; g >>= 1)
    if (positions % g == 0 && grid % (8 * g) == 0) return (unsigned)g;
  return 0;
}

// One stage of compile-time radix B on the tile.  Wave w takes blocks w, w + 4, ...; block
// (a, bp), a < P / (B sp), bp < sp, couples tile rows a B sp + r sp + bp; its values sit at
// prm[(a sp + bp) * BBP ..] (BBP = B * B rounded up to a multiple of 4).
// RP = row pitch of the tile in float2, cidx[cc] = this lane's float2 index inside a tile row
// for each of the NCC column chunks (plain tiles: RP = 64, one chunk, cidx = lane).
template <int B, int RP, int NCC>
__device__ __forceinline__ void col_stage(float2 *tile, const float *prm, const ColOp &op, int P,
                                          int wave, const int (&cidx)[NCC]) {
  constexpr int BBP = (B * B + 3) & ~3;
  const int sp = op.sp;
  const int nblk = P / B;
  const float *region = prm + op.poff[0];
  int a = 0, bp = wave;
  while (bp >= sp) { bp -= sp; ++a; }
  for (int blk = wave; blk < nblk; blk += kColWaves) {
    const int j0 = a * B * sp + bp;
    const float *kb = region + (a * sp + bp) * BBP;
    float K[BBP];
#pragma unroll
    for (int q = 0; q < BBP / 4; ++q) {
      const float4 f = *reinterpret_cast<const float4 *>(kb + 4 * q);
      K[4 * q] = f.x; K[4 * q + 1] = f.y; K[4 * q + 2] = f.z; K[4 * q + 3] = f.w;
    }
#pragma unroll
    for (int cc = 0; cc < NCC; ++cc) {
      float2 x[B], y[B];
#pragma unroll
      for (int r = 0; r < B; ++r) x[r] = tile[(j0 + r * sp) * RP + cidx[cc]];
#pragma unroll
      for (int r2 = 0; r2 < B; ++r2) {
        float ax = 0.f, ay = 0.f;
#pragma unroll
        for (int r = 0; r < B; ++r) {
          ax = fmaf(x[r].x, K[r * B + r2], ax);
          ay = fmaf(x[r].y, K[r * B + r2], ay);
        }
        y[r2] = make_float2(ax, ay);
      }
#pragma unroll
      for (int r = 0; r < B; ++r) tile[(j0 + r * sp) * RP + cidx[cc]] = y[r];
    }
    bp += kColWaves;
    while (bp >= sp) { bp -= sp; ++a; }
  }
}

// K consecutive radix-2 stages on items of 2^K rows (tile rows a 2^K sp + e sp + bp, e < 2^K).
// Sub-stage i pairs e0 (bit dp clear) with e0 + 2^dp; with e0 = eh 2^(dp+1) + el its block is
// number (a 2^(K-dp-1) + eh) * (sp 2^dp) + el sp + bp of the stage's P / 2 blocks in the tile.
// ASC: the sub-stages act on digits 0, 1, .., K-1 in this order, else K-1, .., 0.
template <int K, bool ASC, int RP, int NCC>
__device__ __forceinline__ void col_run2(float2 *tile, const float *prm, const ColOp &op, int P,
                                         int wave, const int (&cidx)[NCC]) {
  constexpr int E = 1 << K;
  const int sp = op.sp;
  const int nitem = P / E;
  int a = 0, bp = wave;
  while (bp >= sp) { bp -= sp; ++a; }
  for (int it = wave; it < nitem; it += kColWaves) {
    const int j0 = a * E * sp + bp;
    float4 kq[K][E / 2];
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const int dp = ASC ? i : K - 1 - i;
      const float *region = prm + op.poff[i];
#pragma unroll
      for (int p = 0; p < E / 2; ++p) {
        const int eh = p >> dp, el = p & ((1 << dp) - 1);
        const int q = ((a << (K - dp - 1)) + eh) * (sp << dp) + el * sp + bp;
        kq[i][p] = *reinterpret_cast<const float4 *>(region + 4 * q);
      }
    }
#pragma unroll
    for (int cc = 0; cc < NCC; ++cc) {
      float2 x[E];
#pragma unroll
      for (int e = 0; e < E; ++e) x[e] = tile[(j0 + e * sp) * RP + cidx[cc]];
#pragma unroll
      for (int i = 0; i < K; ++i) {
        const int dp = ASC ? i : K - 1 - i;
#pragma unroll
        for (int p = 0; p < E / 2; ++p) {
          const int eh = p >> dp, el = p & ((1 << dp) - 1);
          const int e0 = (eh << (dp + 1)) | el, e1 = e0 | (1 << dp);
          const float4 k = kq[i][p];   // k00 k01 k10 k11
          const float2 u = x[e0], v = x[e1];
          x[e0] = make_float2(fmaf(v.x, k.z, u.x * k.x), fmaf(v.y, k.z, u.y * k.x));
          x[e1] = make_float2(fmaf(v.x, k.w, u.x * k.y), fmaf(v.y, k.w, u.y * k.y));
        }
      }
#pragma unroll
      for (int e = 0; e < E; ++e) tile[(j0 + e * sp) * RP + cidx[cc]] = x[e];
    }
    bp += kColWaves;
    while (bp >= sp) { bp -= sp; ++a; }
  }
}

// every step of a pass on the tile in LDS, one barrier after each
template <int RP, int NCC>
__device__ __forceinline__ void col_ops(float2 *tile, const float *prm, const ColPass &cp, int wave,
                                        const int (&cidx)[NCC]) {
  const int P = cp.P;
  for (int oi = 0; oi < cp.nops; ++oi) {
    const ColOp &op = cp.op[oi];
    const bool asc = op.dp[0] == 0;
    if (op.k == 3) {
      if (asc) col_run2<3, true, RP, NCC>(tile, prm, op, P, wave, cidx);
      else col_run2<3, false, RP, NCC>(tile, prm, op, P, wave, cidx);
    } else if (op.k == 2) {
      if (asc) col_run2<2, true, RP, NCC>(tile, prm, op, P, wave, cidx);
      else col_run2<2, false, RP, NCC>(tile, prm, op, P, wave, cidx);
    } else {
      switch (op.b) {
        case 2: col_stage<2, RP, NCC>(tile, prm, op, P, wave, cidx); break;
        case 3: col_stage<3, RP, NCC>(tile, prm, op, P, wave, cidx); break;
        case 4: col_stage<4, RP, NCC>(tile, prm, op, P, wave, cidx); break;
        case 5: col_stage<5, RP, NCC>(tile, prm, op, P, wave, cidx); break;
        case 6: col_stage<6, RP, NCC>(tile, prm, op, P, wave, cidx); break;
        case 7: col_stage<7, RP, NCC>(tile, prm, op, P, wave, cidx); break;
        default: col_stage<8, RP, NCC>(tile, prm, op, P, wave, cidx); break;
      }
    }
    __syncthreads();
  }
}

// A workgroup walks over `tpw` row tiles at one column position; the rows of the next tile are requested into
// registers (up to 32 rows per wave) before the work on the current one starts.
// NRW > 0 (fast variant): 4 <= P <= 4 NRW, every column tile is full and pairs of columns are
// aligned; every wave takes NRW row steps (those past its last row repeat that row) and no
// access is conditional -- the compiler can then count the outstanding loads and stores and
// waits for the rows of the next tile without also waiting for the stores of the previous one
// (vector memory operations retire in order).  NRW == 0: any P <= 128 and ragged column
// tiles, guarded.
template <typename TI, typename TO, bool VEC, int NRW>
__global__ __launch_bounds__(kColThreads) void harp_col_kernel(
    const ColPass *__restrict__ passp, const TI *src, int64_t lds_, TO *dst, int64_t ldd,
    int64_t ncols, unsigned ctiles, unsigned ntiles, unsigned tpw, unsigned xg) {
  // (block-scaled half rows: the exponent bytes of a row follow its ncols halves)
  extern __shared__ float2 tile[];   // [P][64] float2, then npar floats of block values
  const ColPass &cp = *passp;
  const int lane = (int)threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int P = cp.P, S = cp.S;
  constexpr int NR = NRW > 0 ? NRW : kColMaxP / kColWaves;   // rows per wave
  constexpr bool GUARD = (NRW == 0);
  // Unguarded variants (4 <= P <= 4 * NRW): wave w owns the rows w + 4 u, u <= ulast; the steps
  // u > ulast repeat row w + 4 ulast (same address, same LDS slot, same value), so that no
  // access is conditional whatever P is.  The running pointers and LDS slots are clamped
  // per lane (vector arithmetic: one clamp value per tile instead of a scalar per step);
  // P == 4 * NRW takes the plain increments.
  const bool exact = GUARD || (P == kColWaves * NR);
  const int ulast_v = (P - 1 - ((int)threadIdx.x >> 6)) >> 2;   // per lane on purpose

  struct TilePos {
    int hi, lo;
    int64_t row0, col;
    bool v0, v1;
    int eoff;   // bytes from a pair of block-scaled halves to its segment's exponent byte
  };
  auto locate = [&](unsigned t) -> TilePos {
    TilePos tp;
    // tile t = (run * ctiles + ct) * tpw + step: a workgroup stays at one column position and
    // walks down tpw row tiles; consecutive workgroups take neighbouring column positions
    const unsigned u = t / tpw, ct = u % ctiles, rt = (u / ctiles) * tpw + t % tpw;   // rt = hi * S + lo
    tp.hi = (int)(rt / (unsigned)S);
    tp.lo = (int)(rt % (unsigned)S);
    tp.row0 = (int64_t)tp.hi * P * S + tp.lo;
    tp.col = (int64_t)ct * kColCols + 2 * lane;
    tp.v0 = !GUARD || tp.col < ncols;
    tp.v1 = !GUARD || tp.col + 1 < ncols;
    tp.eoff = (int)((ncols - tp.col) * 2 + (tp.col >> 4));
    return tp;
  };
  // Block values of a tile: value e of the pass's list is image[fix[e] + hi * fa[e] + lo * fb[e]]
  // (table built with the plan); thread tid owns e = tid + 256 k and keeps its table entries
  // in registers for the whole launch.
  float *prm = reinterpret_cast<float *>(tile + P * 64);
  // explicitly global: a generic pointer loaded from memory would make these FLAT loads,
  // whose completion order against other memory operations is unknown to the compiler
  typedef const __attribute__((address_space(1))) float *gfloat_t;
  gfloat_t image = (gfloat_t)cp.image;
  const int npar = cp.npar;
  typedef const __attribute__((address_space(1))) uint32_t *gtab_t;
  gtab_t ptab = (gtab_t)cp.ptab;
  unsigned dfix[kColParPerThread], dfa[kColParPerThread], dfb[kColParPerThread];
#pragma unroll
  for (int k = 0; k < kColParPerThread; ++k) {
    const int e = (int)threadIdx.x + kColThreads * k;
    const bool ok = e < npar;
    // entries past the list and padding entries (fa == 0xffffffff) read image[0]: harmless,
    // and it keeps every load unconditional
    const unsigned fa = ok ? ptab[npar + e] : 0xffffffffu;
    const bool real = fa != 0xffffffffu;
    dfix[k] = real ? ptab[e] : 0u;
    dfa[k] = real ? fa : 0u;
    dfb[k] = real ? ptab[2 * npar + e] : 0u;
  }
  float ppre[kColParPerThread];

  ColRaw<TI> pre[NR];
  // per-lane running pointers keep the address arithmetic out of the scalar registers
  auto request = [&](const TilePos &tp) {
#pragma unroll
    for (int k = 0; k < kColParPerThread; ++k)
      ppre[k] = image[dfix[k] + (unsigned)tp.hi * dfa[k] + (unsigned)tp.lo * dfb[k]];
    const TI *rp = src + (tp.row0 + (int64_t)wave * S) * lds_ + tp.col;
    const int64_t step = (int64_t)kColWaves * S * lds_;
    if (exact) {
#pragma unroll
      for (int u = 0; u < NR; ++u) {
        if (!GUARD || wave + kColWaves * u < P) col_load<TI, VEC>(pre[u], rp, tp.v0, tp.v1, tp.eoff);
        rp += step;
      }
    } else {
      const TI *rlast = rp + (int64_t)ulast_v * step;
#pragma unroll
      for (int u = 0; u < NR; ++u) {
        col_load<TI, VEC>(pre[u], rp, tp.v0, tp.v1, tp.eoff);
        rp = (rp + step < rlast) ? rp + step : rlast;
      }
    }
  };

  const unsigned t0 = xcd_grouped(blockIdx.x, xg) * tpw;
  const unsigned t1 = (t0 + tpw < ntiles) ? t0 + tpw : ntiles;
  if (t0 >= t1) return;
  // registers -> LDS: rows and block values of the tile whose request is outstanding
  float2 *tp0 = tile + wave * 64 + lane;
  auto to_lds = [&]() __attribute__((always_inline)) {
    if (exact) {
#pragma unroll
      for (int u = 0; u < NR; ++u)
        if (!GUARD || wave + kColWaves * u < P) tp0[u * (kColWaves * 64)] = col_widen<VEC>(pre[u]);
    } else {
      int su = 0;
#pragma unroll
      for (int u = 0; u < NR; ++u) {
        tp0[su * (kColWaves * 64)] = col_widen<VEC>(pre[u]);
        su = (su + 1 < ulast_v) ? su + 1 : ulast_v;
      }
    }
#pragma unroll
    for (int k = 0; k < kColParPerThread; ++k) prm[(int)threadIdx.x + kColThreads * k] = ppre[k];
  };
  // the stages on the tile in LDS, then LDS -> device memory
  auto work = [&](unsigned t) __attribute__((always_inline)) {
    const TilePos cur = locate(t);
    const int cidx[1] = {lane};
    col_ops<64, 1>(tile, prm, cp, wave, cidx);
    TO *wp = dst + (cur.row0 + (int64_t)wave * S) * ldd + cur.col;
    const int64_t wstep = (int64_t)kColWaves * S * ldd;
    if (exact) {
#pragma unroll
      for (int u = 0; u < NR; ++u) {
        if (!GUARD || wave + kColWaves * u < P)
          col_store<TO, VEC>(wp, tp0[u * (kColWaves * 64)], cur.v0, cur.v1, cur.eoff);
        wp += wstep;
      }
    } else {
      TO *wlast = wp + (int64_t)ulast_v * wstep;
      int su = 0;
#pragma unroll
      for (int u = 0; u < NR; ++u) {
        col_store<TO, VEC>(wp, tp0[su * (kColWaves * 64)], cur.v0, cur.v1, cur.eoff);
        wp = (wp + wstep < wlast) ? wp + wstep : wlast;
        su = (su + 1 < ulast_v) ? su + 1 : ulast_v;
      }
    }
  };
  // Every wait for requested rows inside the loop follows the same sequence (request, stages,
  // stores), so it is a wait for "all but the stores".
  request(locate(t0));
  to_lds();
  for (unsigned t = t0; t + 1 < t1; ++t) {
    __syncthreads();
    request(locate(t + 1));
    work(t);
    __syncthreads();   // every wave has read its rows of the tile back
    to_lds();
  }
  __syncthreads();
  work(t1 - 1);
}

// ------------------------------------------------------------------------------------------
// Column pass of LOGP consecutive radix-2 stages on the tile-row bits 0 .. LOGP-1 (ascending, or
// descending with DESC), P = 2^LOGP rows per tile, with the tile in REGISTERS: a wave owns
// NR = P / 4 rows of the tile (two columns per lane) in one of two layouts,
//     layout A: tile rows w NR + u   (the wave index is the top two bits: stages on bits
//               0 .. LOGP-3 pair rows of the same wave),
//     layout B: tile rows w + 4 u    (the wave index is the low two bits: stages on bits
//               2 .. LOGP-1 pair rows of the same wave),
// so an ascending pass runs LOGP-2 stages in layout A, exchanges the tile through LDS once, and
// runs the last two stages in layout B (a descending pass: LOGP-2 stages in layout B, exchange,
// two in layout A).  One LDS round trip per tile instead of one per group of three stages plus
// the two that staged the tile in and out, three barriers per tile instead of five.  The block
// values travel with the tile as in harp_col_kernel and are read from LDS at wave-uniform
// addresses.  Unguarded tiles only (whole 128-column tiles, aligned pairs).
struct Col2Stages {
  int32_t poff[8];   // offset of stage `bit`'s block values in the tile's list (floats)
};

// one stage on bit UB of the in-wave row index; block of the pair whose lower row is u0:
// number qa + qs * (u0 with bit UB removed), four values k00 k01 k10 k11 at prm4[..]
template <int NR, int UB>
__device__ __forceinline__ void col2_stage(float2 (&x)[NR], const float4 *prm4, int qa, int qs) {
#pragma unroll
  for (int p = 0; p < NR / 2; ++p) {
    const int u0 = ((p >> UB) << (UB + 1)) | (p & ((1 << UB) - 1)), u1 = u0 | (1 << UB);
    const float4 k = prm4[qa + qs * p];   // p is u0 with bit UB removed
    const float2 a = x[u0], b = x[u1];
    x[u0] = make_float2(fmaf(b.x, k.z, a.x * k.x), fmaf(b.y, k.z, a.y * k.x));
    x[u1] = make_float2(fmaf(b.x, k.w, a.x * k.y), fmaf(b.y, k.w, a.y * k.y));
  }
}

// the stages of one layout: FIRST .. FIRST + N - 1 ascending, or FIRST down to FIRST - N + 1
template <int NR, int LOGP, bool LAYOUT_B, int FIRST, int N, bool DESC>
__device__ __forceinline__ void col2_stages(float2 (&x)[NR], const float *prm, const Col2Stages &cs,
                                            int wave) {
  if constexpr (N > 0) {
    constexpr int bit = FIRST;
    constexpr int UB = LAYOUT_B ? bit - 2 : bit;
    const float4 *prm4 = reinterpret_cast<const float4 *>(prm + cs.poff[bit]);
    if constexpr (LAYOUT_B) col2_stage<NR, UB>(x, prm4, wave, 4);
    else col2_stage<NR, UB>(x, prm4, wave * (NR / 2), 1);
    // one stage at a time: hoisting the next stage's block values above this stage's arithmetic
    // costs up to 64 registers, which the 128-row instances do not have
    __builtin_amdgcn_sched_barrier(0);
    col2_stages<NR, LOGP, LAYOUT_B, DESC ? FIRST - 1 : FIRST + 1, N - 1, DESC>(x, prm, cs, wave);
  }
}

template <typename TI, typename TO, int LOGP, bool DESC>
__global__ __launch_bounds__(kColThreads) void harp_col2_kernel(
    const ColPass *__restrict__ passp, const TI *src, int64_t lds_, TO *dst, int64_t ldd,
    int64_t ncols, unsigned ctiles, unsigned ntiles, unsigned tpw, unsigned xg, Col2Stages cs) {
  constexpr int P = 1 << LOGP, NR = P / kColWaves;
  extern __shared__ float2 tile[];   // [P][64] float2, then npar floats of block values
  const ColPass &cp = *passp;
  const int lane = (int)threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int S = cp.S;
  // first and second layout of a tile: ascending A then B, descending B then A
  constexpr bool kFirstB = DESC;
  struct TilePos {
    int hi, lo;
    int64_t row0, col;
    int eoff;
  };
  auto locate = [&](unsigned t) -> TilePos {
    TilePos tp;
    const unsigned u = t / tpw, ct = u % ctiles, rt = (u / ctiles) * tpw + t % tpw;   // rt = hi * S + lo
    tp.hi = (int)(rt / (unsigned)S);
    tp.lo = (int)(rt % (unsigned)S);
    tp.row0 = (int64_t)tp.hi * P * S + tp.lo;
    tp.col = (int64_t)ct * kColCols + 2 * lane;
    tp.eoff = (int)((ncols - tp.col) * 2 + (tp.col >> 4));
    return tp;
  };
  float *prm = reinterpret_cast<float *>(tile + P * 64);
  typedef const __attribute__((address_space(1))) float *gfloat_t;
  typedef const __attribute__((address_space(1))) uint32_t *gtab_t;
  gfloat_t image = (gfloat_t)cp.image;
  gtab_t ptab = (gtab_t)cp.ptab;
  const int npar = cp.npar;
  unsigned dfix[kColParPerThread], dfa[kColParPerThread], dfb[kColParPerThread];
#pragma unroll
  for (int k = 0; k < kColParPerThread; ++k) {
    const int e = (int)threadIdx.x + kColThreads * k;
    const bool ok = e < npar;
    const unsigned fa = ok ? ptab[npar + e] : 0xffffffffu;
    const bool real = fa != 0xffffffffu;
    dfix[k] = real ? ptab[e] : 0u;
    dfa[k] = real ? fa : 0u;
    dfb[k] = real ? ptab[2 * npar + e] : 0u;
  }
  float ppre[kColParPerThread];
  ColRaw<TI> pre[NR];
  // tile row of register u in a layout, as (first row, step) in units of tile rows
  const int firstB = wave, firstA = wave * NR;
  auto request = [&](const TilePos &tp) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < kColParPerThread; ++k)
      ppre[k] = image[dfix[k] + (unsigned)tp.hi * dfa[k] + (unsigned)tp.lo * dfb[k]];
    const TI *rp = src + (tp.row0 + (int64_t)(kFirstB ? firstB : firstA) * S) * lds_ + tp.col;
    const int64_t step = (int64_t)(kFirstB ? kColWaves : 1) * S * lds_;
#pragma unroll
    for (int u = 0; u < NR; ++u) {
      col_load<TI, true>(pre[u], rp, true, true, tp.eoff);
      rp += step;
    }
  };
  const unsigned t0 = xcd_grouped(blockIdx.x, xg) * tpw;
  const unsigned t1 = (t0 + tpw < ntiles) ? t0 + tpw : ntiles;
  if (t0 >= t1) return;
  float2 *colp = tile + lane;
  request(locate(t0));
  for (unsigned t = t0; t < t1; ++t) {
    const TilePos cur = locate(t);
    float2 x[NR];
#pragma unroll
    for (int u = 0; u < NR; ++u) x[u] = col_widen<true>(pre[u]);
#pragma unroll
    for (int k = 0; k < kColParPerThread; ++k) prm[(int)threadIdx.x + kColThreads * k] = ppre[k];
    __syncthreads();   // the tile's block values are in LDS
    // the next tile (after the last one: that tile once more, so that the sequence of requests,
    // stages and stores is the same in every iteration and no access is conditional)
    request(locate(t + 1 < t1 ? t + 1 : t));
    if constexpr (!DESC) col2_stages<NR, LOGP, false, 0, LOGP - 2, false>(x, prm, cs, wave);
    else col2_stages<NR, LOGP, true, LOGP - 1, LOGP - 2, true>(x, prm, cs, wave);
    // exchange: rows of the first layout out, rows of the second layout in
#pragma unroll
    for (int u = 0; u < NR; ++u)
      colp[(kFirstB ? firstB + kColWaves * u : firstA + u) * 64] = x[u];
    __syncthreads();
#pragma unroll
    for (int u = 0; u < NR; ++u)
      x[u] = colp[(kFirstB ? firstA + u : firstB + kColWaves * u) * 64];
    if constexpr (!DESC) col2_stages<NR, LOGP, true, LOGP - 2, 2, false>(x, prm, cs, wave);
    else col2_stages<NR, LOGP, false, 1, 2, true>(x, prm, cs, wave);
    TO *wp = dst + (cur.row0 + (int64_t)(kFirstB ? firstA : firstB) * S) * ldd + cur.col;
    const int64_t wstep = (int64_t)(kFirstB ? 1 : kColWaves) * S * ldd;
#pragma unroll
    for (int u = 0; u < NR; ++u) {
      col_store<TO, true>(wp, x[u], true, true, cur.eoff);
      wp += wstep;
    }
    __syncthreads();   // every wave is done with the block values and the exchange buffer
  }
}

// Column pass fused with ONE stage of the row-side processor (plan_V's streamed stage of radix
// BV on the top digit: it couples the columns lo + r Sv, r < BV, of a row with block lo, and
// commutes with every stage of plan_U).  A tile is P rows x BV segments of 32 columns (row
// pitch BV * 16 float2, two chunks of 64 lanes for BV > 4; lanes past the end of the row
// mirror its last pair -- same address, same value -- so that no access is conditional).  Tiles
// of a workgroup share their column position, so a thread keeps the BV x BV block of its column
// (thread = column j of 32, row group of 8) in registers for the whole launch.  The row stage
// runs on the LDS copy before the column steps.
template <typename TI, typename TO, int BV, int NRW>
__global__ __launch_bounds__(kColThreads, 2) void harp_colrow_kernel(
    const ColPass *__restrict__ passp, const TI *src, int64_t lds_, TO *dst, int64_t ldd,
    const float *__restrict__ vparams, int vnq, int Sv, unsigned nrt, unsigned nct, unsigned tpw,
    unsigned xg) {
  extern __shared__ float2 tile[];   // [P][BV * 16] float2, then the block values of the column steps
  constexpr int RP = BV * 16, NCC = (RP + 63) / 64;
  const ColPass &cp = *passp;
  const int lane = (int)threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int P = cp.P, S = cp.S;   // P == 4 * NRW

  // Workgroup -> (column position ct, tpw consecutive row tiles).  Consecutive workgroups take
  // consecutive column positions, so the 128-byte pieces that are in flight at the same time
  // are neighbours in memory; tiles are numbered t = ct * nrt + rt inside the kernel.
  const unsigned wg = xcd_grouped(blockIdx.x, xg);
  const unsigned ct = wg % nct;
  const unsigned t0 = ct * nrt + (wg / nct) * tpw;
  const int c0 = (int)ct * 32;
  // (lanes past the end of a tile row repeat the pairs of its last eight lanes, so that every
  // aligned group of eight lanes holds one whole 16-column segment)
  int cidx[NCC], eoff[NCC];
  int64_t gcol[NCC];
#pragma unroll
  for (int cc = 0; cc < NCC; ++cc) {
    const int i = cc * 64 + lane;
    cidx[cc] = i < RP ? i : RP - 8 + (lane & 7);
    gcol[cc] = (int64_t)(cidx[cc] / 16) * Sv + c0 + 2 * (cidx[cc] % 16);
    eoff[cc] = (int)(((int64_t)BV * Sv - gcol[cc]) * 2 + (gcol[cc] >> 4));
  }
  // block of the row stage for column c0 + j (value v of block q at vparams[v * vnq + q])
  const int j = (int)threadIdx.x & 31, rg = (int)threadIdx.x >> 5;
  float Kv[BV * BV];
#pragma unroll
  for (int v = 0; v < BV * BV; ++v) Kv[v] = vparams[(size_t)v * vnq + c0 + j];

  float *prm = reinterpret_cast<float *>(tile + P * RP);
  typedef const __attribute__((address_space(1))) float *gfloat_t;
  typedef const __attribute__((address_space(1))) uint32_t *gtab_t;
  gfloat_t image = (gfloat_t)cp.image;
  gtab_t ptab = (gtab_t)cp.ptab;
  const int npar = cp.npar;
  unsigned dfix[kColParPerThread], dfa[kColParPerThread], dfb[kColParPerThread];
#pragma unroll
  for (int k = 0; k < kColParPerThread; ++k) {
    const int e = (int)threadIdx.x + kColThreads * k;
    const bool ok = e < npar;
    const unsigned fa = ok ? ptab[npar + e] : 0xffffffffu;
    const bool real = fa != 0xffffffffu;
    dfix[k] = real ? ptab[e] : 0u;
    dfa[k] = real ? fa : 0u;
    dfb[k] = real ? ptab[2 * npar + e] : 0u;
  }
  float ppre[kColParPerThread];
  ColRaw<TI> pre[NRW][NCC];

  auto request = [&](unsigned t) __attribute__((always_inline)) {
    const unsigned rt = t % nrt;
    const int hi = (int)(rt / (unsigned)S), lo = (int)(rt % (unsigned)S);
    const int64_t row0 = (int64_t)hi * P * S + lo;
#pragma unroll
    for (int k = 0; k < kColParPerThread; ++k)
      ppre[k] = image[dfix[k] + (unsigned)hi * dfa[k] + (unsigned)lo * dfb[k]];
    const TI *rp = src + (row0 + (int64_t)wave * S) * lds_;
    const int64_t step = (int64_t)kColWaves * S * lds_;
#pragma unroll
    for (int u = 0; u < NRW; ++u) {
#pragma unroll
      for (int cc = 0; cc < NCC; ++cc) col_load<TI, true>(pre[u][cc], rp + gcol[cc], true, true, eoff[cc]);
      rp += step;
    }
  };
  float2 *tp0 = tile + wave * RP;
  auto to_lds = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < NRW; ++u)
#pragma unroll
      for (int cc = 0; cc < NCC; ++cc)
        tp0[u * (kColWaves * RP) + cidx[cc]] = col_widen<true>(pre[u][cc]);
#pragma unroll
    for (int k = 0; k < kColParPerThread; ++k) prm[(int)threadIdx.x + kColThreads * k] = ppre[k];
  };
  auto work = [&](unsigned t) __attribute__((always_inline)) {
    // row stage: rows rg, rg + 8, ...; column j of every segment
    float *tf = reinterpret_cast<float *>(tile);
    for (int row = rg; row < P; row += 8) {
      float *rowp = tf + row * (2 * RP) + j;
      float x[BV], y[BV];
#pragma unroll
      for (int r = 0; r < BV; ++r) x[r] = rowp[r * 32];
#pragma unroll
      for (int r2 = 0; r2 < BV; ++r2) {
        float acc = 0.f;
#pragma unroll
        for (int r = 0; r < BV; ++r) acc = fmaf(x[r], Kv[r * BV + r2], acc);
        y[r2] = acc;
      }
#pragma unroll
      for (int r = 0; r < BV; ++r) rowp[r * 32] = y[r];
    }
    __syncthreads();
    col_ops<RP, NCC>(tile, prm, cp, wave, cidx);
    const unsigned rt = t % nrt;
    const int hi = (int)(rt / (unsigned)S), lo = (int)(rt % (unsigned)S);
    const int64_t row0 = (int64_t)hi * P * S + lo;
    TO *wp = dst + (row0 + (int64_t)wave * S) * ldd;
    const int64_t wstep = (int64_t)kColWaves * S * ldd;
#pragma unroll
    for (int u = 0; u < NRW; ++u) {
#pragma unroll
      for (int cc = 0; cc < NCC; ++cc)
        col_store<TO, true>(wp + gcol[cc], tp0[u * (kColWaves * RP) + cidx[cc]], true, true, eoff[cc]);
      wp += wstep;
    }
  };
  request(t0);
  to_lds();
  for (unsigned t = t0; t + 1 < t0 + tpw; ++t) {
    __syncthreads();
    request(t + 1);
    work(t);
    __syncthreads();
    to_lds();
  }
  __syncthreads();
  work(t0 + tpw - 1);
}

// Does the pass consist of radix-2 stages on the tile-row bits 0 .. k-1 in ascending or descending
// order, 32 <= P = 2^k <= 128?  Then it runs with the tile in registers (harp_col2_kernel).
static bool col2_pass(const ColPass &hp, Col2Stages &cs, int &logp, bool &desc) {
  int k = 0;
  while ((1 << k) < hp.P) ++k;
  if ((1 << k) != hp.P || k < 5 || k > 7) return false;
  int bits[8], n = 0;
  for (int oi = 0; oi < hp.nops; ++oi) {
    const ColOp &op = hp.op[oi];
    if (op.b != 2 || op.sp < 1 || (op.sp & (op.sp - 1))) return false;
    int b0 = 0;
    while ((1 << b0) < op.sp) ++b0;
    for (int i = 0; i < op.k; ++i) {
      const int bit = b0 + op.dp[i];
      if (n >= 8 || bit < 0 || bit >= k || (op.poff[i] & 3)) return false;
      bits[n++] = bit;
      cs.poff[bit] = op.poff[i];
    }
  }
  if (n != k) return false;
  bool asc = true, dsc = true;
  for (int i = 0; i < k; ++i) {
    asc = asc && bits[i] == i;
    dsc = dsc && bits[i] == k - 1 - i;
  }
  if (!asc && !dsc) return false;
  logp = k;
  desc = dsc && !asc;
  return true;
}

template <typename TI, typename TO>
struct Col2Types {   // element types the register-tile kernel is built for
  static constexpr bool value =
      (std::is_same<TI, TO>::value && !std::is_same<TI, zh16>::value) ||            // float / bf16 in place
      IsZ16<TI>::value || IsZ16<TO>::value;                                         // the halves
};

template <typename TI, typename TO>
harp_status_t launch_col_tiles(const harp_plan *plan, const ColPass *dpass, const ColPass &hp,
                               const TI *src, int64_t lds_, TO *dst, int64_t ldd, int64_t nrows,
                               int64_t ncols, bool vec, bool fast, hipStream_t stream) {
  const int64_t ctiles = (ncols + kColCols - 1) / kColCols;
  const int64_t tiles = (nrows / hp.P) * ctiles;
  if (tiles <= 0) return HARP_OK;
  if (tiles > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  const size_t shmem = (size_t)hp.P * 64 * sizeof(float2) + (size_t)kColMaxPar * sizeof(float);
  if (shmem > (size_t)plan->lds_bytes) return HARP_ERR_UNSUPPORTED;
  // about four workgroups per resident slot (two 73 KB tiles fit a compute unit), at most 16
  // tiles each (measured flat between 7 and 14 tiles per workgroup; 1 or 56 are 5-9 % slower)
  const int64_t slots = (int64_t)(plan->num_cu > 0 ? plan->num_cu : 256) * 2;
  int64_t tpw = tiles / (slots * 4);
  tpw = std::max<int64_t>(1, std::min<int64_t>(tpw, 16));
  // (a divisor of the number of row tiles: every workgroup walks down whole runs)
  const int64_t nrt = nrows / hp.P;
  while (nrt % tpw != 0) --tpw;
  const int64_t grid = tiles / tpw;
  // 16 neighbouring column tiles share a 128-byte line of exponent bytes
  const unsigned xg = xcd_group_size(ctiles, grid, 16);
  if constexpr (Col2Types<TI, TO>::value) {
    Col2Stages cs{};
    int logp = 0;
    bool desc = false;
    if (fast && col2_pass(hp, cs, logp, desc)) {
      typedef void (*kern2_t)(const ColPass *, const TI *, int64_t, TO *, int64_t, int64_t, unsigned,
                              unsigned, unsigned, unsigned, Col2Stages);
      static const kern2_t table2[6] = {harp_col2_kernel<TI, TO, 5, false>, harp_col2_kernel<TI, TO, 5, true>,
                                        harp_col2_kernel<TI, TO, 6, false>, harp_col2_kernel<TI, TO, 6, true>,
                                        harp_col2_kernel<TI, TO, 7, false>, harp_col2_kernel<TI, TO, 7, true>};
      const int w2 = (logp - 5) * 2 + (desc ? 1 : 0);
      const kern2_t kern2 = table2[w2];
      static thread_local int attr2_done_dev[6] = {-1, -1, -1, -1, -1, -1};   // per instantiation
      if (attr2_done_dev[w2] != plan->device) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern2),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                plan->lds_bytes) != hipSuccess) {
          (void)hipGetLastError();
          return HARP_ERR_DEVICE;
        }
        attr2_done_dev[w2] = plan->device;
      }
      hipLaunchKernelGGL(kern2, dim3((unsigned)grid), dim3(kColThreads), shmem, stream, dpass, src, lds_,
                         dst, ldd, ncols, (unsigned)ctiles, (unsigned)tiles, (unsigned)tpw, xg, cs);
      return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
    }
  }
  typedef void (*kern_t)(const ColPass *, const TI *, int64_t, TO *, int64_t, int64_t, unsigned,
                         unsigned, unsigned, unsigned);
  // unguarded: the variant with the fewest row steps per wave that covers P
  const int which = !fast ? (vec ? 1 : 0)
                          : (hp.P > 64 ? 2 : (hp.P > 32 ? 3 : (hp.P > 16 ? 4 : (hp.P > 8 ? 5 : 6))));
  kern_t kern = nullptr;
  if constexpr (IsZ16<TI>::value || IsZ16<TO>::value) {
    // block-scaled halves exist in the unguarded variants only
    static const kern_t table[7] = {nullptr, nullptr,
                                    harp_col_kernel<TI, TO, true, 32>, harp_col_kernel<TI, TO, true, 16>,
                                    harp_col_kernel<TI, TO, true, 8>,  harp_col_kernel<TI, TO, true, 4>,
                                    harp_col_kernel<TI, TO, true, 2>};
    kern = table[which];
  } else {
    static const kern_t table[7] = {harp_col_kernel<TI, TO, false, 0>, harp_col_kernel<TI, TO, true, 0>,
                                    harp_col_kernel<TI, TO, true, 32>, harp_col_kernel<TI, TO, true, 16>,
                                    harp_col_kernel<TI, TO, true, 8>,  harp_col_kernel<TI, TO, true, 4>,
                                    harp_col_kernel<TI, TO, true, 2>};
    kern = table[which];
  }
  if (!kern) return HARP_ERR_UNSUPPORTED;
  static thread_local int attr_done_dev[7] = {-1, -1, -1, -1, -1, -1, -1};   // per instantiation
  if (attr_done_dev[which] != plan->device) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            plan->lds_bytes) != hipSuccess) {
      (void)hipGetLastError();
      return HARP_ERR_DEVICE;
    }
    attr_done_dev[which] = plan->device;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kColThreads), shmem, stream, dpass, src, lds_,
                     dst, ldd, ncols, (unsigned)ctiles, (unsigned)tiles, (unsigned)tpw, xg);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

// The full column tiles go to the fast variant when the shape allows it, the ragged last
// column tile (and every other shape) to the guarded one.
template <typename TI, typename TO>
harp_status_t launch_col_typed(const harp_plan *plan, const ColPass *dpass, const ColPass &hp,
                               const void *src, int64_t lds_, void *dst, int64_t ldd,
                               int64_t nrows, int64_t ncols, hipStream_t stream) {
  const size_t ei = sizeof(TI), eo = sizeof(TO);
  const bool vec = (ncols % 2 == 0) && (lds_ % 2 == 0) && (ldd % 2 == 0) &&
                   ((uintptr_t)src % (2 * ei) == 0) && ((uintptr_t)dst % (2 * eo) == 0);
  const bool shape_ok = vec && hp.P >= kColWaves && hp.P <= kColMaxP;
  const int64_t full = shape_ok ? (ncols / kColCols) * kColCols : 0;
  if ((IsZ16<TI>::value || IsZ16<TO>::value) && full != ncols) return HARP_ERR_UNSUPPORTED;
  harp_status_t st = HARP_OK;
  if (full > 0)
    st = launch_col_tiles<TI, TO>(plan, dpass, hp, (const TI *)src, lds_, (TO *)dst, ldd, nrows,
                                  full, true, true, stream);
  if (st == HARP_OK && full < ncols)
    st = launch_col_tiles<TI, TO>(plan, dpass, hp, (const TI *)src + full, lds_, (TO *)dst + full,
                                  ldd, nrows, ncols - full, vec, false, stream);
  return st;
}

template <typename TI, typename TO, int BV>
harp_status_t launch_colrow_bv(const harp_plan *plan, const ColPass *dpass, const ColPass &hp,
                               const PassDesc &vp, const TI *src, int64_t lds_, TO *dst,
                               int64_t ldd, int64_t nrows, int64_t ncols, hipStream_t stream) {
  constexpr int RP = BV * 16;
  const int64_t nrt = nrows / hp.P, nct = vp.S / 32;
  const size_t shmem = (size_t)hp.P * RP * sizeof(float2) + (size_t)kColMaxPar * sizeof(float);
  if (shmem > (size_t)plan->lds_bytes) return HARP_ERR_UNSUPPORTED;
  int64_t tpw = 1;
  for (int64_t c = 16; c >= 1; --c)
    if (nrt % c == 0) { tpw = c; break; }
  const int64_t grid = (nrt / tpw) * nct;
  if (grid <= 0 || grid > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  // 2 neighbouring column positions share a line of halves, 64 a line of exponent bytes
  const unsigned xg = xcd_group_size(nct, grid, 64);
  typedef void (*kern_t)(const ColPass *, const TI *, int64_t, TO *, int64_t, const float *, int, int,
                         unsigned, unsigned, unsigned, unsigned);
  const kern_t kern = hp.P == 64 ? (kern_t)harp_colrow_kernel<TI, TO, BV, 16>
                                 : (kern_t)harp_colrow_kernel<TI, TO, BV, 8>;
  static thread_local int attr_done_dev[2] = {-1, -1};   // per instantiation
  const int which = hp.P == 64 ? 0 : 1;
  if (attr_done_dev[which] != plan->device) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            plan->lds_bytes) != hipSuccess) {
      (void)hipGetLastError();
      return HARP_ERR_DEVICE;
    }
    attr_done_dev[which] = plan->device;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kColThreads), shmem, stream, dpass, src, lds_,
                     dst, ldd, vp.params, (int)vp.nq, (int)vp.S, (unsigned)nrt, (unsigned)nct,
                     (unsigned)tpw, xg);
  (void)ncols;
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

template <typename TI, typename TO>
harp_status_t launch_colrow_typed(const harp_plan *plan, const ColPass *dpass, const ColPass &hp,
                                  const PassDesc &vp, const void *src, int64_t lds_, void *dst,
                                  int64_t ldd, int64_t nrows, int64_t ncols, hipStream_t stream) {
  switch (vp.b) {
    case 3: return launch_colrow_bv<TI, TO, 3>(plan, dpass, hp, vp, (const TI *)src, lds_, (TO *)dst, ldd, nrows, ncols, stream);
    case 4: return launch_colrow_bv<TI, TO, 4>(plan, dpass, hp, vp, (const TI *)src, lds_, (TO *)dst, ldd, nrows, ncols, stream);
    case 5: return launch_colrow_bv<TI, TO, 5>(plan, dpass, hp, vp, (const TI *)src, lds_, (TO *)dst, ldd, nrows, ncols, stream);
    case 6: return launch_colrow_bv<TI, TO, 6>(plan, dpass, hp, vp, (const TI *)src, lds_, (TO *)dst, ldd, nrows, ncols, stream);
    case 7: return launch_colrow_bv<TI, TO, 7>(plan, dpass, hp, vp, (const TI *)src, lds_, (TO *)dst, ldd, nrows, ncols, stream);
    case 8: return launch_colrow_bv<TI, TO, 8>(plan, dpass, hp, vp, (const TI *)src, lds_, (TO *)dst, ldd, nrows, ncols, stream);
    default: return HARP_ERR_UNSUPPORTED;
  }
}

}  // namespace

// Host side: group the stages of plan->col[dir] (execution order) into passes and steps, and
// list for every pass the block values a tile needs.  Returns false when the plan has no
// column-mode image (a radix above 8).
bool build_col_passes(const harp_plan *plan, Direction dir, std::vector<ColPassHost> &out) {
  const std::vector<ColStage> &st = plan->col[dir];
  out.clear();
  if (st.empty()) return false;
  const int m = (int)st.size();
  const float *image = st[0].blocks;   // one allocation, stages back to back
  auto padded = [](int b) { return (b * b + 3) & ~3; };
  // Partition of the stages into passes (stages i .. e-1 with prod(b) <= kColMaxP whose block
  // values fit the budget): as few passes as possible -- each one reads and writes the whole
  // matrix -- and among those partitions the one whose smallest tile is tallest (a greedy
  // "fill every pass" split leaves the last pass with whatever remains, down to 2 or 3 rows
  // per tile: 28672 = 7 * 2^12 ended in a pass of P = 2 that took three times as long as the
  // other two together).  Ties go to the taller first pass.
  auto fits = [&](int i0, int e0, int &Pout) {
    int P = 1;
    for (int t = i0; t < e0; ++t) {
      if (P * st[t].b > kColMaxP) return false;
      P *= st[t].b;
    }
    int par = 0;
    for (int t = i0; t < e0; ++t) par += (P / st[t].b) * padded(st[t].b);
    Pout = P;
    return par <= kColMaxPar;
  };
  std::vector<int> best_n(m + 1, 1 << 20), best_min(m + 1, 0), best_e(m + 1, -1);
  best_n[m] = 0;
  best_min[m] = 1 << 30;
  for (int i0 = m - 1; i0 >= 0; --i0) {
    for (int e0 = m; e0 > i0; --e0) {
      int P = 0;
      if (!fits(i0, e0, P) || best_n[e0] >= (1 << 20)) continue;
      const int n = best_n[e0] + 1, mn = std::min(P, best_min[e0]);
      if (n < best_n[i0] || (n == best_n[i0] && mn > best_min[i0])) {
        best_n[i0] = n;
        best_min[i0] = mn;
        best_e[i0] = e0;
      }
    }
  }
  if (best_e[0] < 0) return false;
  int i = 0;
  while (i < m) {
    const int e = best_e[i];
    int P = 0;
    if (e <= i || !fits(i, e, P)) return false;
    int S = st[i].s;
    for (int t = i; t < e; ++t) S = std::min(S, st[t].s);
    out.emplace_back();
    ColPassHost &ph = out.back();
    ph.dev = nullptr;
    ColPass &cp = ph.pass;
    memset(&cp, 0, sizeof(cp));
    cp.P = P;
    cp.S = S;
    cp.image = image;
    std::vector<uint32_t> fix, fa, fb;
    int t = i;
    while (t < e) {
      if (cp.nops >= kColMaxOps) return false;
      ColOp &op = cp.op[cp.nops++];
      op.b = st[t].b;
      int k = 1;
      if (st[t].b == 2) {
        // up to three radix-2 stages on adjacent digits, ascending or descending
        while (k < 3 && t + k < e && st[t + k].b == 2 &&
               (st[t + k].s == st[t + k - 1].s * 2 || st[t + k].s * 2 == st[t + k - 1].s) &&
               (k == 1 || ((st[t + k].s > st[t + k - 1].s) == (st[t + 1].s > st[t].s))))
          ++k;
      }
      op.k = k;
      int smin = st[t].s;
      for (int q = 0; q < k; ++q) smin = std::min(smin, st[t + q].s);
      op.sp = smin / S;
      for (int q = 0; q < k; ++q) {
        const ColStage &cs = st[t + q];
        int dp = 0;
        while ((smin << dp) < cs.s) ++dp;
        op.dp[q] = dp;
        op.poff[q] = (int32_t)fix.size();
        // blocks of this stage inside a tile: number j = a' s' + beta' (s' = s / S) is block
        // c = hi (P / b) S + lo + a' s + beta' S of the stage
        const int b = cs.b, bb = b * b, bbp = padded(b), sp = cs.s / S;
        const uint32_t off = (uint32_t)(cs.blocks - image);
        for (int j = 0; j < P / b; ++j) {
          const int ap = j / sp, bt = j % sp;
          for (int v = 0; v < bbp; ++v) {
            const bool real = v < bb;
            fix.push_back(real ? off + (uint32_t)((int64_t)ap * cs.s + (int64_t)bt * S) * bb + v : 0u);
            fa.push_back(real ? (uint32_t)P * (uint32_t)S * (uint32_t)b : 0xffffffffu);
            fb.push_back(real ? (uint32_t)bb : 0u);
          }
        }
      }
      t += k;
    }
    cp.npar = (int32_t)fix.size();
    if (cp.npar > kColMaxPar) return false;
    ph.ptab = fix;
    ph.ptab.insert(ph.ptab.end(), fa.begin(), fa.end());
    ph.ptab.insert(ph.ptab.end(), fb.begin(), fb.end());
    i = e;
  }
  return true;
}

harp_status_t launch_col_pass(const harp_plan *plan, const ColPass *dpass, const ColPass &hp,
                              const void *src,
                              int64_t lds_, harp_dtype_t dt_src, void *dst, int64_t ldd,
                              harp_dtype_t dt_dst, int64_t nrows, int64_t ncols,
                              hipStream_t stream) {
  if (nrows % hp.P != 0) return HARP_ERR_INVALID_ARG;
  const bool zs = (int)dt_src == kDtZ16, zd = (int)dt_dst == kDtZ16;
  if (zs && zd)
    return launch_col_typed<zh16, zh16>(plan, dpass, hp, src, lds_, dst, ldd, nrows, ncols, stream);
  if (zs && dt_dst == HARP_BF16)
    return launch_col_typed<zh16, uint16_t>(plan, dpass, hp, src, lds_, dst, ldd, nrows, ncols, stream);
  if (zd && dt_src == HARP_BF16)
    return launch_col_typed<uint16_t, zh16>(plan, dpass, hp, src, lds_, dst, ldd, nrows, ncols, stream);
  if (zs || zd) return HARP_ERR_UNSUPPORTED;
  if (dt_src == HARP_F32 && dt_dst == HARP_F32)
    return launch_col_typed<float, float>(plan, dpass, hp, src, lds_, dst, ldd, nrows, ncols, stream);
  if (dt_src == HARP_BF16 && dt_dst == HARP_F32)
    return launch_col_typed<uint16_t, float>(plan, dpass, hp, src, lds_, dst, ldd, nrows, ncols, stream);
  if (dt_src == HARP_F32 && dt_dst == HARP_BF16)
    return launch_col_typed<float, uint16_t>(plan, dpass, hp, src, lds_, dst, ldd, nrows, ncols, stream);
  return launch_col_typed<uint16_t, uint16_t>(plan, dpass, hp, src, lds_, dst, ldd, nrows, ncols, stream);
}

// A column pass with block-scaled halves on either side runs in the unguarded variants only:
// whole 128-column tiles, aligned pairs, 4 <= P <= 128.
bool col_z16_supported(const ColPass &hp, const void *src, int64_t lds_, const void *dst,
                       int64_t ldd, int64_t nrows, int64_t ncols) {
  if (ncols % kColCols != 0 || nrows % hp.P != 0) return false;
  if (hp.P < kColWaves || hp.P > kColMaxP) return false;
  if (lds_ % 2 || ldd % 2 || (uintptr_t)src % 4 || (uintptr_t)dst % 4) return false;
  return true;
}

// Would this pass run with the tile in registers (harp_col2_kernel) on whole column tiles?
bool col_pass_in_registers(const ColPass &hp, int64_t ncols) {
  Col2Stages cs{};
  int logp = 0;
  bool desc = false;
  return ncols % kColCols == 0 && col2_pass(hp, cs, logp, desc);
}

// The fused launch applies when: the column pass has exactly 32 or 64 rows per tile; the row
// stage is a dense small-radix stage (3..8) on the top digit of a processor on ncols coordinates
// whose stride is a multiple of 32; pairs of columns are aligned in both matrices.
bool colrow_supported(const harp_plan *plan, const ColPass &hp, const PassDesc &vp, const void *src,
                      int64_t lds_, harp_dtype_t dt_src, const void *dst, int64_t ldd,
                      harp_dtype_t dt_dst, int64_t nrows, int64_t ncols) {
  if (hp.P != 64 && hp.P != 32) return false;
  if (hp.P == 64 && vp.b == 8) return false;   // would not fit 256 vector registers
  if (nrows % hp.P != 0) return false;
  if (vp.kind != PASS_SMALL || vp.b < 3 || vp.b > 8) return false;
  if ((int64_t)vp.b * vp.S != ncols || vp.nq != vp.S || vp.S % 32 != 0) return false;
  const size_t ei = dt_src == HARP_F32 ? 4 : 2, eo = dt_dst == HARP_F32 ? 4 : 2;
  if (lds_ % 2 || ldd % 2 || (uintptr_t)src % (2 * ei) || (uintptr_t)dst % (2 * eo)) return false;
  // block-scaled halves: the workspace of a bf16 matrix (the other side bf16 or halves as well)
  const bool zs = (int)dt_src == kDtZ16, zd = (int)dt_dst == kDtZ16;
  if ((zs && dt_dst == HARP_F32) || (zd && dt_src == HARP_F32)) return false;
  const size_t shmem = (size_t)hp.P * vp.b * 16 * sizeof(float2) + (size_t)kColMaxPar * sizeof(float);
  return shmem <= (size_t)plan->lds_bytes;
}

harp_status_t launch_colrow_pass(const harp_plan *plan, const ColPass *dpass, const ColPass &hp,
                                 const PassDesc &vp, const void *src, int64_t lds_,
                                 harp_dtype_t dt_src, void *dst, int64_t ldd, harp_dtype_t dt_dst,
                                 int64_t nrows, int64_t ncols, hipStream_t stream) {
  if ((int)dt_src == kDtZ16 && dt_dst == HARP_BF16)
    return launch_colrow_typed<zh16, uint16_t>(plan, dpass, hp, vp, src, lds_, dst, ldd, nrows, ncols, stream);
  if (dt_src == HARP_BF16 && (int)dt_dst == kDtZ16)
    return launch_colrow_typed<uint16_t, zh16>(plan, dpass, hp, vp, src, lds_, dst, ldd, nrows, ncols, stream);
  if ((int)dt_src == kDtZ16 && (int)dt_dst == kDtZ16)
    return launch_colrow_typed<zh16, zh16>(plan, dpass, hp, vp, src, lds_, dst, ldd, nrows, ncols, stream);
  if ((int)dt_src == kDtZ16 || (int)dt_dst == kDtZ16) return HARP_ERR_UNSUPPORTED;
  if (dt_src == HARP_F32 && dt_dst == HARP_F32)
    return launch_colrow_typed<float, float>(plan, dpass, hp, vp, src, lds_, dst, ldd, nrows, ncols, stream);
  if (dt_src == HARP_BF16 && dt_dst == HARP_F32)
    return launch_colrow_typed<uint16_t, float>(plan, dpass, hp, vp, src, lds_, dst, ldd, nrows, ncols, stream);
  if (dt_src == HARP_F32 && dt_dst == HARP_BF16)
    return launch_colrow_typed<float, uint16_t>(plan, dpass, hp, vp, src, lds_, dst, ldd, nrows, ncols, stream);
  return launch_colrow_typed<uint16_t, uint16_t>(plan, dpass, hp, vp, src, lds_, dst, ldd, nrows, ncols, stream);
}

}  // namespace harp
