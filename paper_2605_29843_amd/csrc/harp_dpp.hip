// Two-group row pipeline for radix-2 chains in the two-shear form on rows, or contiguous row
// chunks, of D = 4096 coordinates (twelve stages): eight of the twelve digits are exchanged
// inside a wave with DPP operands of the fused multiply-add itself, so a row makes ONE round
// trip through LDS and the stride permutations of Eq. (7) cost no instruction at all.
//
// A thread always owns 16 consecutive coordinates (digits 0..3, in registers).  The other eight
// digits are spread over lanes and waves in one of two layouts:
//
//   layout L (low):   the four DPP digits are 4..7, lane bits 4,5 are digits 8,9, the wave is 10,11
//   layout H (high):  the four DPP digits are 8..11, lane bits 4,5 are digits 4,5, the wave is 6,7
//
// A DPP digit p of a lane's 16-lane row is reached by one lane permutation that is an
// involution: p = 0 quad_perm [1,0,3,2] (lane ^ 1), p = 1 quad_perm [2,3,0,1] (lane ^ 2),
// p = 2 row_half_mirror (lane ^ 7), p = 3 row_ror:8 (lane ^ 8).  These four masks are linearly
// independent over GF(2), so the low four lane bits l map one-to-one onto digit values
// e = (l0 ^ l2, l1 ^ l2, l2, l3), and a stage on DPP digit p is, for every register j,
//
//        x[j] <- x[j] + f[j] * x[j] of the partner lane          (v_fmac_f32 with a DPP src0)
//
// with f the shear factor of the lane's own coordinate (m10/m00 for the member with digit value
// 0, m01/m11 for the other; Alg. 1's block multiply in the scaled form the plan builder
// derives).  A stage on a register digit pairs registers instead.
//
// Forward programs (digits ascending): group A loads the row in layout L, runs digits 0..3 in
// registers and 4..7 by DPP, writes LDS; group B reads in layout H, runs 8..11 by DPP (the
// program's last stage, when it is in this chunk, is a dense 2x2 carrying every pending scale)
// and stores.  Transposed programs (digits descending): group A loads in layout H and runs
// 11..8, group B reads in layout L, runs 7..4 by DPP and 3..0 in registers, and stores.  Rows
// move in pairs, group B one pair behind group A, one workgroup barrier per pair:
// ceil(rows / 2) + 1 steps per tile.  Every parameter is read from device memory once per
// workgroup, 16 bytes per lane and 1 KB of consecutive addresses per wave instruction (the
// image is laid out in thread order by the plan builder), and stays in registers.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "harp_internal.h"

namespace harp {

namespace {

constexpr int kLogD = 12, kD = 1 << kLogD, kTG = kD / 16;       // 256 threads per group
constexpr int kPlane = 260;                                       // 256 floats + 4 of padding
constexpr int kRowBuf = (kD / 256) * kPlane;                      // floats per buffered row
// The same kernel on rows or chunks of 2048 coordinates (eleven stages; LOGD = 11): 128 threads
// per group; layout L as above with one wave bit (digit 10); layout H: the DPP digits are 8, 9,
// 10 and (unused as a stage) 4, lane bits 4,5 are digits 5,6, the wave is digit 7.  Group A of a
// forward program still runs digits 0..7, group B the three digits 8..10; transposed: A runs
// 10..8, B 7..0.  And on 1024 coordinates (ten stages; LOGD = 10): one wave per group; layout H:
// the DPP digits are 8, 9 and (unused as stages) 4, 5, lane bits 4,5 are digits 6,7.
template <int LOGD>
struct Geo {
  static constexpr int D = 1 << LOGD, TG = D / 16, ROWBUF = (D / 256) * kPlane;
  static constexpr int NHI = LOGD - 8;   // stages on the digits above 7
};
constexpr int kPrefetchPairs = 1;
constexpr int kSleepB = 0;

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  bf2 v;
  v.x = (__bf16)lo;
  v.y = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

// Segment (run of 16 coordinates) of thread (wave w, lane l) in the two layouts.
template <int LOGD = 12>
__device__ __forceinline__ unsigned seg_of(bool high, unsigned w, unsigned l) {
  const unsigned low4 = l & 15u;
  const unsigned e = low4 ^ (((low4 >> 2) & 1u) * 3u);   // digit values of the four DPP digits
  if (LOGD == 11)
    return high ? ((e >> 3) | ((l >> 4) << 1) | (w << 3) | ((e & 7u) << 4))
                : (e | ((l >> 4) << 4) | (w << 6));
  if (LOGD == 10)
    return high ? ((e >> 2) | ((l >> 4) << 2) | ((e & 3u) << 4)) : (e | ((l >> 4) << 4));
  return high ? ((l >> 4) | (w << 2) | (e << 4)) : (e | ((l >> 4) << 4) | (w << 6));
}

// LDS position (floats) of 16-byte piece k of segment s: planes of 256 coordinates 260 floats
// apart, the four pieces of a segment permuted by two parity bits of the segment index.  With
// this placement the 16-byte accesses of both layouts are free of bank conflicts, for 32 banks
// served 8 lanes at a time and for 64 banks served 16 lanes at a time.
__device__ __forceinline__ unsigned lds_piece(unsigned s, unsigned k) {
  const unsigned g = ((s >> 2) & 1u) | ((((s >> 1) ^ (s >> 3)) & 1u) << 1);
  return (s >> 4) * kPlane + 16u * (s & 15u) + 4u * (k ^ g);
}

// ---- stages ------------------------------------------------------------------------------
// eight registers of one DPP shear stage: x[O + i] += f[O + i] * partner(x[O + i]).  The block
// opens with two wait states: the instruction before it may have written the first register a
// DPP operand reads (VALU write -> DPP read needs two), and the compiler cannot see into the
// block.  Inside, a register's read is at least eight instructions after its last write.
#define HARP_DPP_FMAC8(CTRL, X, F, O)                                                   \
  asm volatile("s_nop 1\n\t"                                                             \
               "v_fmac_f32_dpp %0, %0, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"      \
               "v_fmac_f32_dpp %1, %1, %9 " CTRL " row_mask:0xf bank_mask:0xf\n\t"      \
               "v_fmac_f32_dpp %2, %2, %10 " CTRL " row_mask:0xf bank_mask:0xf\n\t"     \
               "v_fmac_f32_dpp %3, %3, %11 " CTRL " row_mask:0xf bank_mask:0xf\n\t"     \
               "v_fmac_f32_dpp %4, %4, %12 " CTRL " row_mask:0xf bank_mask:0xf\n\t"     \
               "v_fmac_f32_dpp %5, %5, %13 " CTRL " row_mask:0xf bank_mask:0xf\n\t"     \
               "v_fmac_f32_dpp %6, %6, %14 " CTRL " row_mask:0xf bank_mask:0xf\n\t"     \
               "v_fmac_f32_dpp %7, %7, %15 " CTRL " row_mask:0xf bank_mask:0xf"         \
               : "+v"(X[O + 0]), "+v"(X[O + 1]), "+v"(X[O + 2]), "+v"(X[O + 3]),         \
                 "+v"(X[O + 4]), "+v"(X[O + 5]), "+v"(X[O + 6]), "+v"(X[O + 7])          \
               : "v"(F[O + 0]), "v"(F[O + 1]), "v"(F[O + 2]), "v"(F[O + 3]),             \
                 "v"(F[O + 4]), "v"(F[O + 5]), "v"(F[O + 6]), "v"(F[O + 7]))

// eight registers of the dense DPP stage: m[O + i] += g[O + i] * partner(x[O + i])
#define HARP_DPP_FMAC8_SRC(CTRL, M, X, G, O)                                            \
  asm volatile("s_nop 1\n\t"                                                             \
               "v_fmac_f32_dpp %0, %8, %16 " CTRL " row_mask:0xf bank_mask:0xf\n\t"     \
               "v_fmac_f32_dpp %1, %9, %17 " CTRL " row_mask:0xf bank_mask:0xf\n\t"     \
               "v_fmac_f32_dpp %2, %10, %18 " CTRL " row_mask:0xf bank_mask:0xf\n\t"    \
               "v_fmac_f32_dpp %3, %11, %19 " CTRL " row_mask:0xf bank_mask:0xf\n\t"    \
               "v_fmac_f32_dpp %4, %12, %20 " CTRL " row_mask:0xf bank_mask:0xf\n\t"    \
               "v_fmac_f32_dpp %5, %13, %21 " CTRL " row_mask:0xf bank_mask:0xf\n\t"    \
               "v_fmac_f32_dpp %6, %14, %22 " CTRL " row_mask:0xf bank_mask:0xf\n\t"    \
               "v_fmac_f32_dpp %7, %15, %23 " CTRL " row_mask:0xf bank_mask:0xf"        \
               : "+v"(M[O + 0]), "+v"(M[O + 1]), "+v"(M[O + 2]), "+v"(M[O + 3]),         \
                 "+v"(M[O + 4]), "+v"(M[O + 5]), "+v"(M[O + 6]), "+v"(M[O + 7])          \
               : "v"(X[O + 0]), "v"(X[O + 1]), "v"(X[O + 2]), "v"(X[O + 3]),             \
                 "v"(X[O + 4]), "v"(X[O + 5]), "v"(X[O + 6]), "v"(X[O + 7]),             \
                 "v"(G[O + 0]), "v"(G[O + 1]), "v"(G[O + 2]), "v"(G[O + 3]),             \
                 "v"(G[O + 4]), "v"(G[O + 5]), "v"(G[O + 6]), "v"(G[O + 7]))

template <int P>
__device__ __forceinline__ void dpp_shear(float (&x)[16], const float (&f)[16]) {
  if (P == 0) {
    HARP_DPP_FMAC8("quad_perm:[1,0,3,2]", x, f, 0);
    HARP_DPP_FMAC8("quad_perm:[1,0,3,2]", x, f, 8);
  } else if (P == 1) {
    HARP_DPP_FMAC8("quad_perm:[2,3,0,1]", x, f, 0);
    HARP_DPP_FMAC8("quad_perm:[2,3,0,1]", x, f, 8);
  } else if (P == 2) {
    HARP_DPP_FMAC8("row_half_mirror", x, f, 0);
    HARP_DPP_FMAC8("row_half_mirror", x, f, 8);
  } else {
    HARP_DPP_FMAC8("row_ror:8", x, f, 0);
    HARP_DPP_FMAC8("row_ror:8", x, f, 8);
  }
}

// dense 2x2 on DPP digit P: x <- ms * x + mo * partner(x)
template <int P>
__device__ __forceinline__ void dpp_dense(float (&x)[16], const float (&ms)[16], const float (&mo)[16]) {
  float m[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) m[j] = x[j] * ms[j];
  if (P == 0) {
    HARP_DPP_FMAC8_SRC("quad_perm:[1,0,3,2]", m, x, mo, 0);
    HARP_DPP_FMAC8_SRC("quad_perm:[1,0,3,2]", m, x, mo, 8);
  } else if (P == 1) {
    HARP_DPP_FMAC8_SRC("quad_perm:[2,3,0,1]", m, x, mo, 0);
    HARP_DPP_FMAC8_SRC("quad_perm:[2,3,0,1]", m, x, mo, 8);
  } else if (P == 2) {
    HARP_DPP_FMAC8_SRC("row_half_mirror", m, x, mo, 0);
    HARP_DPP_FMAC8_SRC("row_half_mirror", m, x, mo, 8);
  } else {
    HARP_DPP_FMAC8_SRC("row_ror:8", m, x, mo, 0);
    HARP_DPP_FMAC8_SRC("row_ror:8", m, x, mo, 8);
  }
#pragma unroll
  for (int j = 0; j < 16; ++j) x[j] = m[j];
}

// shear stage on register digit BP: pairs (j, j | 1 << BP)
template <int BP>
__device__ __forceinline__ void reg_shear(float (&x)[16], const float (&f)[16]) {
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const int j0 = ((p >> BP) << (BP + 1)) | (p & ((1 << BP) - 1)), j1 = j0 | (1 << BP);
    const float x0 = x[j0], x1 = x[j1];
    x[j0] = fmaf(f[j0], x1, x0);
    x[j1] = fmaf(f[j1], x0, x1);
  }
}

template <int BP>
__device__ __forceinline__ void reg_dense(float (&x)[16], const float (&ms)[16], const float (&mo)[16]) {
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const int j0 = ((p >> BP) << (BP + 1)) | (p & ((1 << BP) - 1)), j1 = j0 | (1 << BP);
    const float x0 = x[j0], x1 = x[j1];
    x[j0] = fmaf(mo[j0], x1, ms[j0] * x0);
    x[j1] = fmaf(mo[j1], x0, ms[j1] * x1);
  }
}

// ---- element I/O: 16 consecutive coordinates of a row ---------------------------------------
template <typename T>
struct Seg16;
template <>
struct Seg16<uint16_t> {
  static constexpr int NRAW = 8;
  __device__ static __forceinline__ void load(const uint16_t *p, uint32_t (&raw)[NRAW]) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint4 v = reinterpret_cast<const uint4 *>(p)[h];
      raw[4 * h] = v.x; raw[4 * h + 1] = v.y; raw[4 * h + 2] = v.z; raw[4 * h + 3] = v.w;
    }
  }
  __device__ static __forceinline__ void unpack(const uint32_t (&raw)[NRAW], float (&x)[16]) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      x[2 * m] = __uint_as_float(raw[m] << 16);
      x[2 * m + 1] = __uint_as_float(raw[m] & 0xffff0000u);
    }
  }
  __device__ static __forceinline__ void store(uint16_t *p, const float (&x)[16]) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
      reinterpret_cast<uint4 *>(p)[h] =
          make_uint4(cvt_pk_bf16(x[8 * h], x[8 * h + 1]), cvt_pk_bf16(x[8 * h + 2], x[8 * h + 3]),
                     cvt_pk_bf16(x[8 * h + 4], x[8 * h + 5]), cvt_pk_bf16(x[8 * h + 6], x[8 * h + 7]));
  }
};
template <>
struct Seg16<float> {
  static constexpr int NRAW = 16;
  __device__ static __forceinline__ void load(const float *p, uint32_t (&raw)[NRAW]) {
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const uint4 v = reinterpret_cast<const uint4 *>(p)[h];
      raw[4 * h] = v.x; raw[4 * h + 1] = v.y; raw[4 * h + 2] = v.z; raw[4 * h + 3] = v.w;
    }
  }
  __device__ static __forceinline__ void unpack(const uint32_t (&raw)[NRAW], float (&x)[16]) {
#pragma unroll
    for (int e = 0; e < 16; ++e) x[e] = __uint_as_float(raw[e]);
  }
  __device__ static __forceinline__ void store(float *p, const float (&x)[16]) {
#pragma unroll
    for (int h = 0; h < 4; ++h)
      reinterpret_cast<float4 *>(p)[h] = make_float4(x[4 * h], x[4 * h + 1], x[4 * h + 2], x[4 * h + 3]);
  }
};

// 16 block-scaled halves = one aligned segment of the intermediate of a split program; ep = the
// segment's exponent byte
template <>
struct Seg16<zh16> {
  static constexpr int NRAW = 9;
  __device__ static __forceinline__ void load(const zh16 *p, const uint8_t *ep, uint32_t (&raw)[NRAW]) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint4 v = reinterpret_cast<const uint4 *>(p)[h];
      raw[4 * h] = v.x; raw[4 * h + 1] = v.y; raw[4 * h + 2] = v.z; raw[4 * h + 3] = v.w;
    }
    raw[8] = *ep;
  }
  __device__ static __forceinline__ void unpack(const uint32_t (&raw)[NRAW], float (&x)[16]) {
    const float sc = z16_up(raw[8]);
#pragma unroll
    for (int m = 0; m < 8; ++m) z16_unpack(raw[m], sc, x[2 * m], x[2 * m + 1]);
  }
  __device__ static __forceinline__ void store(zh16 *p, uint8_t *ep, const float (&x)[16]) {
    float mx = fabsf(x[0]);
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(mx, fabsf(x[e]));
    const uint32_t ex = z16_exponent(mx);
    const float f = z16_down(ex);
#pragma unroll
    for (int h = 0; h < 2; ++h)
      reinterpret_cast<uint4 *>(p)[h] =
          make_uint4(z16_pack(x[8 * h] * f, x[8 * h + 1] * f), z16_pack(x[8 * h + 2] * f, x[8 * h + 3] * f),
                     z16_pack(x[8 * h + 4] * f, x[8 * h + 5] * f), z16_pack(x[8 * h + 6] * f, x[8 * h + 7] * f));
    *ep = (uint8_t)ex;
  }
};

// NS stages' parameters of this thread: value q of piece k of stage e at img[((e * 4 + k) * 256 + t) * 4 + q]
template <int NS, int TG = kTG>
__device__ __forceinline__ void load_params(const float *__restrict__ img, int t, float (&f)[NS][16]) {
  const float4 *p = reinterpret_cast<const float4 *>(img);
#pragma unroll
  for (int e = 0; e < NS; ++e) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float4 v = p[(e * 4 + k) * TG + t];
      f[e][4 * k] = v.x; f[e][4 * k + 1] = v.y; f[e][4 * k + 2] = v.z; f[e][4 * k + 3] = v.w;
    }
    // keep the requests in stage order (vector loads return in order, and the first step waits
    // for each stage's values only when it reaches that stage)
    __builtin_amdgcn_sched_barrier(0);
  }
}

__device__ __forceinline__ void lds_put(float *row, unsigned s, const float (&x)[16]) {
#pragma unroll
  for (int k = 0; k < 4; ++k)
    *reinterpret_cast<float4 *>(row + lds_piece(s, k)) =
        make_float4(x[4 * k], x[4 * k + 1], x[4 * k + 2], x[4 * k + 3]);
}
__device__ __forceinline__ void lds_get(const float *row, unsigned s, float (&x)[16]) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const float4 v = *reinterpret_cast<const float4 *>(row + lds_piece(s, k));
    x[4 * k] = v.x; x[4 * k + 1] = v.y; x[4 * k + 2] = v.z; x[4 * k + 3] = v.w;
  }
}

// ---- group A: device memory -> stages -> LDS -----------------------------------------------
// forward: eight shear stages (register digits 0..3, DPP digits 0..3 of layout L);
// transposed: four shear stages (DPP digits 3..0 of layout H)
template <bool TRN, int LOGD = 12>
__device__ __forceinline__ void stages_A(float (&x)[16], const float (&f)[TRN ? LOGD - 8 : 8][16]) {
  if constexpr (!TRN) {
    reg_shear<0>(x, f[0]);
    reg_shear<1>(x, f[1]);
    reg_shear<2>(x, f[2]);
    reg_shear<3>(x, f[3]);
    dpp_shear<0>(x, f[4]);
    dpp_shear<1>(x, f[5]);
    dpp_shear<2>(x, f[6]);
    dpp_shear<3>(x, f[7]);
  } else if constexpr (LOGD == 11) {
    dpp_shear<2>(x, f[0]);
    dpp_shear<1>(x, f[1]);
    dpp_shear<0>(x, f[2]);
  } else if constexpr (LOGD == 10) {
    dpp_shear<1>(x, f[0]);
    dpp_shear<0>(x, f[1]);
  } else {
    dpp_shear<3>(x, f[0]);
    dpp_shear<2>(x, f[1]);
    dpp_shear<1>(x, f[2]);
    dpp_shear<0>(x, f[3]);
  }
}

// PF = pairs of rows requested ahead of the one being computed
// Et (block-scaled half rows only): exponent byte of the chunk's first segment in the tile's
// first row; the rows' exponents are 2 ldx bytes apart.
template <typename TI, bool TRN, int PF, int LOGD = 12>
__device__ __forceinline__ void group_A(const float *__restrict__ img, int t, float *buf,
                                         const TI *__restrict__ Xt, int64_t ldx, int nr,
                                         const uint8_t *__restrict__ Et) {
  constexpr int NS = TRN ? LOGD - 8 : 8;
  constexpr int kRowBuf = Geo<LOGD>::ROWBUF;
  using In = Seg16<TI>;
  constexpr int NRAW = In::NRAW;
  constexpr bool kZ = std::is_same<TI, zh16>::value;
  const unsigned s = seg_of<LOGD>(TRN, (unsigned)t >> 6, (unsigned)t & 63u);
  const TI *xp = Xt + 16u * s;
  const int last = nr - 1;
  // rows past the end of the tile read its last row again (same address, nothing depends on it),
  // so that every load is unconditional
  auto row_ptr = [&](int r) { return xp + (int64_t)(r < last ? r : last) * ldx; };
  auto load_row = [&](int r, uint32_t (&raw)[NRAW]) {
    if constexpr (kZ) In::load(row_ptr(r), Et + (int64_t)(r < last ? r : last) * (2 * ldx) + s, raw);
    else In::load(row_ptr(r), raw);
  };
  uint32_t pre[2 * PF][NRAW];
  load_row(0, pre[0]);
  load_row(1, pre[1]);
  __builtin_amdgcn_sched_barrier(0);
  float f[NS][16];
  load_params<NS, Geo<LOGD>::TG>(img, t, f);
#pragma unroll
  for (int q = 1; q < PF; ++q) {
    load_row(2 * q, pre[2 * q]);
    load_row(2 * q + 1, pre[2 * q + 1]);
  }
  const int npairs = (nr + 1) >> 1;
  auto step = [&](int k, int q) {
    float xa[16], xb[16];
    In::unpack(pre[2 * q], xa);
    In::unpack(pre[2 * q + 1], xb);
    load_row(2 * (k + PF), pre[2 * q]);
    load_row(2 * (k + PF) + 1, pre[2 * q + 1]);
    float *b = buf + (k & 1) * (2 * kRowBuf);
    stages_A<TRN, LOGD>(xa, f);
    lds_put(b, s, xa);
    stages_A<TRN, LOGD>(xb, f);
    lds_put(b + kRowBuf, s, xb);
  };
  // The first PF steps stand outside the loop: straight-line code after the loads above, in
  // which the compiler waits for each stage's parameters only when that stage needs them, so
  // the first rows are transformed while the rest of the parameter image is still arriving.
#pragma unroll
  for (int q = 0; q < PF; ++q) {
    if (q > npairs) break;
    if (q < npairs) step(q, q);
    __syncthreads();
  }
  for (int k0 = PF; k0 <= npairs; k0 += PF) {
#pragma unroll
    for (int q = 0; q < PF; ++q) {
      const int k = k0 + q;
      if (k > npairs) break;
      if (k < npairs) step(k, q);
      __syncthreads();
    }
  }
}

// ---- group B: LDS -> stages -> device memory ------------------------------------------------
// forward: DPP digits 0..3 of layout H (the last one dense with LD); transposed: DPP digits
// 3..0 of layout L, then register digits 3..0 (the last one dense; a transposed program
// always ends inside the chunk)
template <bool TRN, bool LD, int LOGD = 12>
struct ParamsB {
  static constexpr int NS = (TRN ? 8 : LOGD - 8) - (LD ? 1 : 0);
  float f[NS][16];
  float md[2][16];            // dense stage (LD only): own-coordinate and partner factors
};

template <bool TRN, bool LD, int LOGD = 12>
__device__ __forceinline__ void stages_B(float (&x)[16], const ParamsB<TRN, LD, LOGD> &pb) {
  if constexpr (!TRN && LOGD == 11) {
    dpp_shear<0>(x, pb.f[0]);
    dpp_shear<1>(x, pb.f[1]);
    if constexpr (LD) dpp_dense<2>(x, pb.md[0], pb.md[1]);
    else dpp_shear<2>(x, pb.f[2]);
  } else if constexpr (!TRN && LOGD == 10) {
    dpp_shear<0>(x, pb.f[0]);
    if constexpr (LD) dpp_dense<1>(x, pb.md[0], pb.md[1]);
    else dpp_shear<1>(x, pb.f[1]);
  } else if constexpr (!TRN) {
    dpp_shear<0>(x, pb.f[0]);
    dpp_shear<1>(x, pb.f[1]);
    dpp_shear<2>(x, pb.f[2]);
    if constexpr (LD) dpp_dense<3>(x, pb.md[0], pb.md[1]);
    else dpp_shear<3>(x, pb.f[3]);
  } else {
    dpp_shear<3>(x, pb.f[0]);
    dpp_shear<2>(x, pb.f[1]);
    dpp_shear<1>(x, pb.f[2]);
    dpp_shear<0>(x, pb.f[3]);
    reg_shear<3>(x, pb.f[4]);
    reg_shear<2>(x, pb.f[5]);
    reg_shear<1>(x, pb.f[6]);
    if constexpr (LD) reg_dense<0>(x, pb.md[0], pb.md[1]);
    else reg_shear<0>(x, pb.f[7]);
  }
}

template <typename TO, bool TRN, bool LD, int LOGD = 12>
__device__ __forceinline__ void group_B(const float *__restrict__ img, int t, const float *buf,
                                         TO *__restrict__ Yt, int64_t ldy, int nr,
                                         uint8_t *__restrict__ Et) {
  using Out = Seg16<TO>;
  constexpr bool kZ = std::is_same<TO, zh16>::value;
  constexpr int kRowBuf = Geo<LOGD>::ROWBUF, kTG = Geo<LOGD>::TG;
  using PB = ParamsB<TRN, LD, LOGD>;
  const unsigned s = seg_of<LOGD>(!TRN, (unsigned)t >> 6, (unsigned)t & 63u);
  TO *yp = Yt + 16u * s;
  PB pb;
  // Group A's requests go first: this group needs its parameters one step later, and both share
  // the compute unit's one load path.
  __builtin_amdgcn_s_sleep(kSleepB);
  load_params<PB::NS, kTG>(img, t, pb.f);
  if constexpr (LD) load_params<2, kTG>(img + PB::NS * 16 * kTG, t, pb.md);
  const int npairs = (nr + 1) >> 1;
  auto step = [&](int k) {
    const float *b = buf + ((k - 1) & 1) * (2 * kRowBuf);
    const int r0 = 2 * (k - 1);
    float xa[16], xb[16];
    lds_get(b, s, xa);
    lds_get(b + kRowBuf, s, xb);
    stages_B<TRN, LD, LOGD>(xa, pb);
    if constexpr (kZ) Out::store(yp + (int64_t)r0 * ldy, Et + (int64_t)r0 * (2 * ldy) + s, xa);
    else Out::store(yp + (int64_t)r0 * ldy, xa);
    stages_B<TRN, LD, LOGD>(xb, pb);
    if (r0 + 1 < nr) {
      if constexpr (kZ) Out::store(yp + (int64_t)(r0 + 1) * ldy, Et + (int64_t)(r0 + 1) * (2 * ldy) + s, xb);
      else Out::store(yp + (int64_t)(r0 + 1) * ldy, xb);
    }
  };
  // steps 0 (nothing to do yet) and 1 outside the loop: straight-line code in which each stage
  // waits for its own parameters only
  __syncthreads();
  if (npairs >= 1) {
    step(1);
    __syncthreads();
  }
  for (int k = 2; k <= npairs; ++k) {
    step(k);
    __syncthreads();
  }
}

// Workgroup -> (chunk kch, tile of R rows).  imgA / imgB: the two groups' parameter images of
// chunk 0; chunk kch's follow at kch * strideA / strideB floats.
template <typename TI, typename TO, bool TRN, bool LD, int LOGD = 12>
__global__ __launch_bounds__(2 * Geo<LOGD>::TG) void harp_dpp_kernel(const TI *__restrict__ X, int64_t ldx,
                                                           TO *__restrict__ Y, int64_t ldy,
                                                           int64_t n, int R, int nchunk,
                                                           const float *__restrict__ imgA,
                                                           const float *__restrict__ imgB,
                                                           int64_t strideA, int64_t strideB) {
  constexpr int kD = Geo<LOGD>::D, kTG = Geo<LOGD>::TG;
  __shared__ float buf[4 * Geo<LOGD>::ROWBUF];
  const int g = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kTG);   // wave-uniform
  const int t = (int)threadIdx.x % kTG;
  const int kch = (int)(blockIdx.x % (unsigned)nchunk);
  const int64_t row0 = (int64_t)(blockIdx.x / (unsigned)nchunk) * R;
  const int nr = (int)((n - row0 < R) ? (n - row0) : R);
  // block-scaled half rows: d halves, then the row's exponent bytes (one per 16 coordinates)
  const int64_t d = (int64_t)nchunk * kD;
  if (g == 0)
    group_A<TI, TRN, kPrefetchPairs, LOGD>(imgA + kch * strideA, t, buf, X + row0 * ldx + (int64_t)kch * kD, ldx, nr,
                                           reinterpret_cast<const uint8_t *>(X + row0 * ldx + d) + kch * (kD / 16));
  else
    group_B<TO, TRN, LD, LOGD>(imgB + kch * strideB, t, buf, Y + row0 * ldy + (int64_t)kch * kD, ldy, nr,
                               reinterpret_cast<uint8_t *>(Y + row0 * ldy + d) + kch * (kD / 16));
}

// ------------------------------------------------------------------------------------------
// Transposed split programs whose one streamed stage is a dense stage of radix B = 2, 3 or 5 on the
// digit above the chunk (8192 = 4096 * 2, 12288 = 4096 * 3, 20480 = 4096 * 5): that stage runs first, so it is
// executed on the way in instead of taking its own trip through a float32 intermediate in
// device memory.  For the workgroup's chunk k the first group reads its 16 coordinates from ALL
// B chunks of the row and forms z[i] = sum_j x[j * 4096 + i] * K_i[j][k] with the B factors of
// each coordinate in registers (the block of Alg. 1's stage belongs to the coordinate inside
// the chunk), then goes on as group A above.  The row is read B times, but the B workgroups of
// one row tile are numbered so that they run on one XCD next to each other and share that
// XCD's L2 (measured: 1.4 times the input fetched from device memory at B = 7), and nothing but
// bf16 rows ever crosses device memory.  Radix 7 (14336, 28672) was built and measured too
// (its 112 + 64 factors need the shear factors in LDS): 131 us against 132 us for the two
// launches at 2048 x 28672 -- in this layout the four lanes of a quad read addresses 512 bytes
// apart, so a wave's 16-byte loads cost four tag look-ups per quad instead of one, and 2 * B of
// them per row saturate the compute unit's load path; radix 3 gains 30 % (52.9 -> 36.8 us at
// 2048 x 12288), radix 5 14 %.
//
// A whole row of requests is in flight per thread (ring of B segments): slot (j, h) is refilled
// with the same piece of the next row as soon as it has been consumed.
template <int B, int LOGD = 12>
__device__ __forceinline__ void group_TA(const float *__restrict__ imgT, const float *__restrict__ imgA,
                                          int t, float *buf, const uint16_t *__restrict__ Xt,
                                          int64_t ldx, int nr) {
  constexpr int kD = Geo<LOGD>::D, kTG = Geo<LOGD>::TG, kRowBuf = Geo<LOGD>::ROWBUF;
  const unsigned s = seg_of<LOGD>(true, (unsigned)t >> 6, (unsigned)t & 63u);
  const unsigned voff = 32u * s;   // byte offset of the thread's segment inside a chunk
  const int last = nr - 1;
  // half h of chunk j of row r; rows past the end of the tile repeat its last row.  The address
  // is a wave-uniform base (scalar registers) plus the one per-lane offset above.
  auto half_ld = [&](int r, int h, int j) -> uint4 {
    const char *base = reinterpret_cast<const char *>(Xt + (int64_t)(r < last ? r : last) * ldx + j * kD) + 16 * h;
    return *reinterpret_cast<const uint4 *>(base + voff);
  };
  // ring of the B chunks of one row (both halves): slot (j, h) is refilled with the same piece
  // of the next row as soon as it has been consumed, so a whole row of requests is in flight
  uint4 raw[B][2];
#pragma unroll
  for (int j = 0; j < B; ++j) {
    raw[j][0] = half_ld(0, 0, j);
    raw[j][1] = half_ld(0, 1, j);
  }
  __builtin_amdgcn_sched_barrier(0);
  float T[B][16];
  load_params<B, kTG>(imgT, t, T);
  float f[LOGD - 8][16];
  load_params<LOGD - 8, kTG>(imgA, t, f);
  const int npairs = (nr + 1) >> 1;
  auto one_row = [&](int r, float *dst) {
    float z[16];
#pragma unroll
    for (int j = 0; j < B; ++j)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint32_t w[4] = {raw[j][h].x, raw[j][h].y, raw[j][h].z, raw[j][h].w};
        raw[j][h] = half_ld(r + 1, h, j);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const float x0 = __uint_as_float(w[m] << 16), x1 = __uint_as_float(w[m] & 0xffff0000u);
          const int i = 8 * h + 2 * m;
          z[i] = (j == 0) ? x0 * T[0][i] : fmaf(x0, T[j][i], z[i]);
          z[i + 1] = (j == 0) ? x1 * T[0][i + 1] : fmaf(x1, T[j][i + 1], z[i + 1]);
        }
        // one chunk at a time: without this the scheduler unpacks several chunks ahead and
        // the B = 7 instance no longer fits 256 registers
        __builtin_amdgcn_sched_barrier(0);
      }
    stages_A<true, LOGD>(z, f);
    lds_put(dst, s, z);
  };
  for (int k = 0; k <= npairs; ++k) {
    if (k < npairs) {
      float *b = buf + (k & 1) * (2 * kRowBuf);
      one_row(2 * k, b);
      one_row(2 * k + 1, b + kRowBuf);
    }
    __syncthreads();
  }
}

// Workgroup b -> XCD b mod 8; the B workgroups of one row tile sit on one XCD, consecutive in
// its dispatch order: i = b / 8, chunk k = i mod B, tile = (i / B) * 8 + (b mod 8).  The grid
// is padded to a multiple of 8 * B workgroups; those past the last tile leave at once.
// imgT: [B chunks][B][4 pieces][256 threads][4] factors; imgA / imgB as in harp_dpp_kernel.
template <int B, int LOGD = 12>
__global__ __launch_bounds__(2 * Geo<LOGD>::TG) void harp_dpp_top_kernel(const uint16_t *__restrict__ X,
                                                               int64_t ldx, uint16_t *__restrict__ Y,
                                                               int64_t ldy, int64_t n, int R,
                                                               const float *__restrict__ imgT,
                                                               const float *__restrict__ imgA,
                                                               const float *__restrict__ imgB,
                                                               int64_t strideA, int64_t strideB) {
  constexpr int kD = Geo<LOGD>::D, kTG = Geo<LOGD>::TG;
  __shared__ float buf[4 * Geo<LOGD>::ROWBUF];
  const int g = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kTG);   // wave-uniform
  const int t = (int)threadIdx.x % kTG;
  const unsigned xcd = blockIdx.x & 7u, i = blockIdx.x >> 3;
  const int kch = (int)(i % (unsigned)B);
  const int64_t tile = (int64_t)(i / (unsigned)B) * 8 + xcd;
  const int64_t row0 = tile * R;
  if (row0 >= n) return;
  const int nr = (int)((n - row0 < R) ? (n - row0) : R);
  if (g == 0)
    group_TA<B, LOGD>(imgT + (int64_t)kch * (B * 16 * kTG), imgA + kch * strideA, t, buf, X + row0 * ldx,
                      ldx, nr);
  else
    group_B<uint16_t, true, true, LOGD>(imgB + kch * strideB, t, buf,
                                        Y + row0 * ldy + (int64_t)kch * kD, ldy, nr, nullptr);
}

template <typename TI, typename TO, int LOGD = 12>
harp_status_t launch_dpp_io(const DppImage &di, const void *X, int64_t ldx, void *Y, int64_t ldy,
                            int64_t n, int R, int nchunk, hipStream_t stream) {
  const int64_t tiles = ((n + R - 1) / R) * nchunk;
  if (tiles > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)tiles), block(2 * Geo<LOGD>::TG);
  const float *a = di.img, *b = di.img + di.offB;
#define HARP_DPP_LAUNCH(TRN_, LD_)                                                                    \
  hipLaunchKernelGGL((harp_dpp_kernel<TI, TO, TRN_, LD_, LOGD>), grid, block, 0, stream, (const TI *)X, \
                     ldx, (TO *)Y, ldy, n, R, nchunk, a, b, di.strideA, di.strideB)
  if (di.trn) {
    if (!di.ld) return HARP_ERR_UNSUPPORTED;
    HARP_DPP_LAUNCH(true, true);
  } else if (di.ld) {
    HARP_DPP_LAUNCH(false, true);
  } else {
    HARP_DPP_LAUNCH(false, false);
  }
#undef HARP_DPP_LAUNCH
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

}  // namespace

// Thread (group, t) of the kernel owns this segment; the plan builder lays the image out with it.
unsigned dpp_segment_of(bool high_layout, unsigned t, int logd) {
  const unsigned w = t >> 6, l = t & 63u;
  const unsigned low4 = l & 15u;
  const unsigned e = low4 ^ (((low4 >> 2) & 1u) * 3u);
  if (logd == 11)
    return high_layout ? ((e >> 3) | ((l >> 4) << 1) | (w << 3) | ((e & 7u) << 4))
                       : (e | ((l >> 4) << 4) | (w << 6));
  if (logd == 10)
    return high_layout ? ((e >> 2) | ((l >> 4) << 2) | ((e & 3u) << 4)) : (e | ((l >> 4) << 4));
  return high_layout ? ((l >> 4) | (w << 2) | (e << 4)) : (e | ((l >> 4) << 4) | (w << 6));
}

bool dpp_supported(const harp_plan *plan, const DppImage &di, int chunk, const void *X, int64_t ldx,
                   harp_dtype_t dt_in, const void *Y, int64_t ldy, harp_dtype_t dt_out) {
  if (plan->algo == HARP_ALGO_GENERIC || !di.img || chunk != (1 << di.logd)) return false;
  // bf16 rows on both sides only: a thread's 16 float32 coordinates are four 16-byte pieces 64
  // bytes apart from its neighbours', the one slow access pattern of this chip (measured:
  // float32 rows 18.2 -> 21.7 us, the float32 intermediate of a 28672-wide split program
  // 250 -> 297 us); those cases keep the three-group kernel, which re-lays rows out in LDS
  // (block-scaled halves, the intermediate of a split program for bf16 callers, are 32 bytes per
  // lane like bf16: written going up, read going down)
  const bool plain = (dt_in == HARP_BF16 && dt_out == HARP_BF16);
  const bool zout = (dt_in == HARP_BF16 && (int)dt_out == kDtZ16 && !di.trn && di.ld);
  const bool zin = ((int)dt_in == kDtZ16 && dt_out == HARP_BF16 && di.trn);
  if (!plain && !zout && !zin) return false;
  // 16-byte row accesses for either element type
  if ((ldx % 8) || (ldy % 8) || ((uintptr_t)X % 16) || ((uintptr_t)Y % 16)) return false;
  return true;
}

harp_status_t launch_dpp_kernel(const harp_plan *plan, const DppImage &di, const void *X,
                                int64_t ldx, harp_dtype_t dt_in, void *Y, int64_t ldy,
                                harp_dtype_t dt_out, int64_t n, int R, hipStream_t stream) {
  const int nchunk = (int)(plan->d >> di.logd);
#define HARP_DPP_BY_TYPE(LOGD_)                                                                 \
  do {                                                                                          \
    if (dt_in == HARP_BF16 && dt_out == HARP_BF16)                                              \
      return launch_dpp_io<uint16_t, uint16_t, LOGD_>(di, X, ldx, Y, ldy, n, R, nchunk, stream); \
    if (dt_in == HARP_BF16 && (int)dt_out == kDtZ16 && !di.trn && di.ld)                        \
      return launch_dpp_io<uint16_t, zh16, LOGD_>(di, X, ldx, Y, ldy, n, R, nchunk, stream);    \
    if ((int)dt_in == kDtZ16 && dt_out == HARP_BF16 && di.trn)                                  \
      return launch_dpp_io<zh16, uint16_t, LOGD_>(di, X, ldx, Y, ldy, n, R, nchunk, stream);    \
    return HARP_ERR_UNSUPPORTED;                                                                \
  } while (0)
  if (di.logd == 11) HARP_DPP_BY_TYPE(11);
  if (di.logd == 10) HARP_DPP_BY_TYPE(10);
#undef HARP_DPP_BY_TYPE
  if (dt_in == HARP_BF16 && dt_out == HARP_BF16)
    return launch_dpp_io<uint16_t, uint16_t>(di, X, ldx, Y, ldy, n, R, nchunk, stream);
  if (dt_in == HARP_BF16 && (int)dt_out == kDtZ16 && !di.trn && di.ld)
    return launch_dpp_io<uint16_t, zh16>(di, X, ldx, Y, ldy, n, R, nchunk, stream);
  if ((int)dt_in == kDtZ16 && dt_out == HARP_BF16 && di.trn)
    return launch_dpp_io<zh16, uint16_t>(di, X, ldx, Y, ldy, n, R, nchunk, stream);
  return HARP_ERR_UNSUPPORTED;   // see dpp_supported
}

bool dpp_top_supported(const harp_plan *plan, const DppImage &di, const void *X, int64_t ldx,
                       harp_dtype_t dt_in, const void *Y, int64_t ldy, harp_dtype_t dt_out) {
  if (plan->algo == HARP_ALGO_GENERIC || !di.img || di.topB == 0 || !di.trn || !di.ld ||
      (di.logd != 12 && di.logd != 11 && di.logd != 10))
    return false;
  if (dt_in != HARP_BF16 || dt_out != HARP_BF16) return false;
  if ((ldx % 8) || (ldy % 8) || ((uintptr_t)X % 16) || ((uintptr_t)Y % 16)) return false;
  // the groups read every chunk of a row before the last one of it is written, but a workgroup
  // of another chunk may already have stored its part of the same row: not in place
  if (X == Y) return false;
  return true;
}

harp_status_t launch_dpp_top_kernel(const harp_plan *plan, const DppImage &di, const void *X,
                                    int64_t ldx, void *Y, int64_t ldy, int64_t n, int R,
                                    hipStream_t stream) {
  const int B = di.topB;
  if (plan->d != ((int64_t)B << di.logd)) return HARP_ERR_UNSUPPORTED;
  const int64_t tiles = (n + R - 1) / R;
  const int64_t wgs = ((tiles + 7) / 8) * 8 * B;
  if (wgs > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)wgs), block(2 * (1 << (di.logd - 4)));
  const float *a = di.img, *b = di.img + di.offB, *tt = di.img + di.offT;
#define HARP_DPP_TOP(B_, L_)                                                                            \
  hipLaunchKernelGGL((harp_dpp_top_kernel<B_, L_>), grid, block, 0, stream, (const uint16_t *)X, ldx, \
                     (uint16_t *)Y, ldy, n, R, tt, a, b, di.strideA, di.strideB)
#define HARP_DPP_TOP_B(L_)                       \
  switch (B) {                                   \
    case 2: HARP_DPP_TOP(2, L_); break;          \
    case 3: HARP_DPP_TOP(3, L_); break;          \
    case 5: HARP_DPP_TOP(5, L_); break;          \
    default: return HARP_ERR_UNSUPPORTED;        \
  }
  if (di.logd == 12) { HARP_DPP_TOP_B(12) }
  else if (di.logd == 11) { HARP_DPP_TOP_B(11) }
  else { HARP_DPP_TOP_B(10) }
#undef HARP_DPP_TOP_B
#undef HARP_DPP_TOP
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

}  // namespace harp
