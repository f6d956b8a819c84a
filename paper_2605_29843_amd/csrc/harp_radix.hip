// Tile kernel for chains of equal small radices (all stages radix 4 or all radix 8, e.g. the
// 4 x radix-8 schedule of d = 4096): rows, or contiguous row chunks, of B^m coordinates.
//
// A dense B x B block costs B^2 parameters per B coordinates, so the parameters of a whole row
// (0.5 MB for 4096 = 8^4) do not fit the register file of a compute unit: they are re-read for
// every tile of R rows, and the kernel is organised to hide that.  A workgroup keeps R <= 8 rows
// in LDS as float32; in stage t thread q owns block c = q of the stage (Alg. 1: coordinates
// base(q) + j * S, S = B^t the stride of the stage), holds its B^2 values in registers for all
// rows of the tile, and while it works on stage t the loads of its block of stage t+1 are
// already in flight.  The first stage takes its inputs straight from device memory (all rows of
// the tile requested at once) and the last stage stores straight to device memory, so a tile
// makes m - 1 LDS round trips and m barriers.  LDS rows are padded by 8 floats per 64 so that
// the stride-B accesses of the second stage fall into distinct banks.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "harp_internal.h"

namespace harp {

namespace {

constexpr int kRMax = 8;   // rows per tile (compile-time bound of the prefetch registers)

typedef const __attribute__((address_space(1))) float *gfloat_t;

__device__ __forceinline__ int lds_pos(int i) { return i + ((i >> 6) << 3); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  bf2 v;
  v.x = (__bf16)lo;
  v.y = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

// B elements of one block of one row, from device memory: contiguous (S == 1) or at stride S
template <typename T, int B>
struct BlockIo;

template <int B>
struct BlockIo<uint16_t, B> {
  static constexpr int NRAW = B;   // contiguous: B / 2 dwords used; strided: one element per dword
  template <bool C>
  __device__ static __forceinline__ void load(const uint16_t *p, int S, uint32_t (&raw)[NRAW]) {
    if (C) {
      if (B == 8) {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        raw[0] = v.x; raw[1] = v.y; raw[2] = v.z; raw[3] = v.w;
      } else {
        const uint2 v = *reinterpret_cast<const uint2 *>(p);
        raw[0] = v.x; raw[1] = v.y;
      }
    } else {
#pragma unroll
      for (int j = 0; j < B; ++j) raw[j] = p[(size_t)j * S];
    }
  }
  template <bool C>
  __device__ static __forceinline__ void unpack(const uint32_t (&raw)[NRAW], float (&x)[B]) {
    if (C) {
#pragma unroll
      for (int m = 0; m < B / 2; ++m) {
        x[2 * m] = __uint_as_float(raw[m] << 16);
        x[2 * m + 1] = __uint_as_float(raw[m] & 0xffff0000u);
      }
    } else {
#pragma unroll
      for (int j = 0; j < B; ++j) x[j] = __uint_as_float(raw[j] << 16);
    }
  }
  template <bool C>
  __device__ static __forceinline__ void store(uint16_t *p, int S, const float (&y)[B]) {
    uint32_t w[(B + 1) / 2];
#pragma unroll
    for (int m = 0; m < (B + 1) / 2; ++m)
      w[m] = pack_bf16(y[2 * m], (2 * m + 1 < B) ? y[2 * m + 1] : 0.0f);
    if (C) {
      if (B == 8) *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
      else *reinterpret_cast<uint2 *>(p) = make_uint2(w[0], w[1]);
    } else {
#pragma unroll
      for (int j = 0; j < B; ++j)
        p[(size_t)j * S] = (uint16_t)((j & 1) ? (w[j / 2] >> 16) : (w[j / 2] & 0xffffu));
    }
  }
};

template <int B>
struct BlockIo<float, B> {
  static constexpr int NRAW = B;
  template <bool C>
  __device__ static __forceinline__ void load(const float *p, int S, uint32_t (&raw)[NRAW]) {
    if (C) {
#pragma unroll
      for (int h = 0; h < B / 4; ++h) {
        const uint4 v = *reinterpret_cast<const uint4 *>(p + 4 * h);
        raw[4 * h] = v.x; raw[4 * h + 1] = v.y; raw[4 * h + 2] = v.z; raw[4 * h + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int j = 0; j < B; ++j) raw[j] = __float_as_uint(p[(size_t)j * S]);
    }
  }
  template <bool C>
  __device__ static __forceinline__ void unpack(const uint32_t (&raw)[NRAW], float (&x)[B]) {
#pragma unroll
    for (int j = 0; j < B; ++j) x[j] = __uint_as_float(raw[j]);
  }
  template <bool C>
  __device__ static __forceinline__ void store(float *p, int S, const float (&y)[B]) {
    if (C) {
#pragma unroll
      for (int h = 0; h < B / 4; ++h)
        *reinterpret_cast<float4 *>(p + 4 * h) =
            make_float4(y[4 * h], y[4 * h + 1], y[4 * h + 2], y[4 * h + 3]);
    } else {
#pragma unroll
      for (int j = 0; j < B; ++j) p[(size_t)j * S] = y[j];
    }
  }
};

// y = x * K (row vector on the left), K row-major in prm
template <int B>
__device__ __forceinline__ void block_mul(const float (&x)[B], const float (&prm)[B * B],
                                          float (&y)[B]) {
#pragma unroll
  for (int c = 0; c < B; ++c) y[c] = x[0] * prm[c];
#pragma unroll
  for (int r = 1; r < B; ++r)
#pragma unroll
    for (int c = 0; c < B; ++c) y[c] = fmaf(x[r], prm[r * B + c], y[c]);
}

// ---- run-time reconstruction of a block from its int8 codes --------------------------------
// (appendix "Int8 storage of HARP parameters"; block definition of Sec. 3: B = Q(theta) G,
// Q = (I + A)^{-1} (I - A) for the skew-symmetric A whose strict upper triangle, row by row, is
// a = s q.)  Q = 2 (I + A)^{-1} - I; the inverse by in-place Gauss-Jordan elimination without
// pivoting: every leading principal minor of I + A is positive because its symmetric part is I.
// With the Hadamard mixer G = H / sqrt(B): row i of Q G = (2 / sqrt(B)) WHT(row i of the
// inverse) - H[i] / sqrt(B).
template <int B>
struct Q8Raw {
  static constexpr int NW = (B == 8) ? 8 : 2;   // dwords of codes, sign bits and padding
  uint32_t w[NW];
  float s;
};

template <int B>
__device__ __forceinline__ void q8_request(const PassDesc &pd, unsigned qg, Q8Raw<B> &raw) {
  const unsigned nq = (unsigned)pd.nq;
  const char *base = reinterpret_cast<const char *>(pd.q8);
  if (B == 8) {
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const uint4 v = *reinterpret_cast<const uint4 *>(base + ((size_t)k * nq + qg) * 16);
      raw.w[4 * k] = v.x; raw.w[4 * k + 1] = v.y; raw.w[4 * k + 2] = v.z; raw.w[4 * k + 3] = v.w;
    }
    raw.s = *reinterpret_cast<const float *>(base + (size_t)nq * 32 + (size_t)qg * 4);
  } else {
    const uint2 v = *reinterpret_cast<const uint2 *>(base + (size_t)qg * 8);
    raw.w[0] = v.x; raw.w[1] = v.y;
    raw.s = *reinterpret_cast<const float *>(base + (size_t)nq * 8 + (size_t)qg * 4);
  }
}

// prm[r * B + c] = entry [r][c] of the block as this direction uses it (TRN: the transpose),
// with the signs of stage 0 on the rows of the forward block
template <int B, bool TRN>
__device__ __forceinline__ void q8_rebuild(const Q8Raw<B> &raw, int flags, float (&prm)[B * B]) {
  constexpr int NP = B * (B - 1) / 2;
  float m[B][B];
  {
    int k = 0;
#pragma unroll
    for (int i = 0; i < B; ++i) {
      m[i][i] = 1.0f;
#pragma unroll
      for (int j = i + 1; j < B; ++j, ++k) {
        const int code = (int)(int8_t)(raw.w[k >> 2] >> (8 * (k & 3)));
        const float a = raw.s * (float)code;
        m[i][j] = a;
        m[j][i] = -a;
      }
    }
  }
#pragma unroll
  for (int c = 0; c < B; ++c) {
    const float p = 1.0f / m[c][c];
    m[c][c] = 1.0f;
#pragma unroll
    for (int j = 0; j < B; ++j) m[c][j] *= p;
#pragma unroll
    for (int r = 0; r < B; ++r) {
      if (r == c) continue;
      const float f = m[r][c];
      m[r][c] = 0.0f;
#pragma unroll
      for (int j = 0; j < B; ++j) m[r][j] = fmaf(-f, m[c][j], m[r][j]);
    }
  }
  if (flags & 1) {
    // Walsh-Hadamard transform of every row (Sylvester order), then the affine map above
    const float g = (B == 8) ? 0.35355339059327379f : 0.5f;   // 1 / sqrt(B)
#pragma unroll
    for (int i = 0; i < B; ++i) {
#pragma unroll
      for (int h = 1; h < B; h <<= 1)
#pragma unroll
        for (int j = 0; j < B; ++j)
          if (!(j & h)) {
            const float u = m[i][j], v = m[i][j | h];
            m[i][j] = u + v;
            m[i][j | h] = u - v;
          }
#pragma unroll
      for (int j = 0; j < B; ++j)
        m[i][j] = fmaf(m[i][j], 2.0f * g, (__builtin_popcount(i & j) & 1) ? g : -g);
    }
  } else {
#pragma unroll
    for (int i = 0; i < B; ++i)
#pragma unroll
      for (int j = 0; j < B; ++j) m[i][j] = fmaf(m[i][j], 2.0f, i == j ? -1.0f : 0.0f);
  }
  if (flags & 2) {
    const uint32_t bits = (raw.w[NP >> 2] >> (8 * (NP & 3))) & 0xffu;
#pragma unroll
    for (int i = 0; i < B; ++i) {
      const uint32_t flip = ((bits >> i) & 1u) << 31;
#pragma unroll
      for (int j = 0; j < B; ++j) m[i][j] = __uint_as_float(__float_as_uint(m[i][j]) ^ flip);
    }
  }
#pragma unroll
  for (int r = 0; r < B; ++r)
#pragma unroll
    for (int c = 0; c < B; ++c) prm[r * B + c] = TRN ? m[c][r] : m[r][c];
}

// One stage on the rows of the tile.  MODE 0: inputs from the prefetched device-memory words
// `raw`, outputs to LDS; 1: LDS in place; 2: inputs from LDS, outputs to device memory.
// CONTIG: the stage's stride is 1 (16-byte accesses); it can only be the first or last stage.
// nqa: blocks of the stage in one chunk row; with GUARD, threads whose block index is beyond
// it idle (kernels whose stages have different block counts).
template <typename TI, typename TO, int B, int BPT, int MODE, bool CONTIG, bool GUARD = false>
__device__ __forceinline__ void radix_pass(float *tile, int dpad, int nr, int S, int tid, int NT,
                                           int nqa, const float (&prm)[BPT][B * B],
                                           const uint32_t (&raw)[kRMax][BPT][B], TO *Yt,
                                           int64_t ldy) {
  using In = BlockIo<TI, B>;
  using Out = BlockIo<TO, B>;
  int base[BPT];
#pragma unroll
  for (int u = 0; u < BPT; ++u) {
    const int q = tid + u * NT, hi = q / S, lo = q - hi * S;
    base[u] = hi * B * S + lo;
  }
  // rows in pairs: the LDS reads of both rows are issued before the first is computed, and the
  // writes of the first are in flight while the second is computed
#pragma unroll
  for (int r = 0; r < kRMax; r += 2) {
    if (r < nr) {
      const bool two = r + 1 < nr;
      float *trow[2] = {tile + r * dpad, tile + (two ? r + 1 : r) * dpad};
#pragma unroll
      for (int u = 0; u < BPT; ++u) {
        if (GUARD && tid + u * NT >= nqa) continue;
        float x[2][B], y[B];
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          if (MODE == 0) {
            In::template unpack<CONTIG>(raw[r + h2][u], x[h2]);
          } else if (CONTIG) {
#pragma unroll
            for (int h = 0; h < B / 4; ++h) {
              const float4 f =
                  *reinterpret_cast<const float4 *>(trow[h2] + lds_pos(base[u] + 4 * h));
              x[h2][4 * h] = f.x; x[h2][4 * h + 1] = f.y; x[h2][4 * h + 2] = f.z; x[h2][4 * h + 3] = f.w;
            }
          } else {
#pragma unroll
            for (int j = 0; j < B; ++j) x[h2][j] = trow[h2][lds_pos(base[u] + j * S)];
          }
        }
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          if (h2 == 1 && !two) break;
          block_mul<B>(x[h2], prm[u], y);
          if (MODE == 2) {
            Out::template store<CONTIG>(Yt + (int64_t)(r + h2) * ldy + base[u], S, y);
          } else if (CONTIG) {
#pragma unroll
            for (int h = 0; h < B / 4; ++h)
              *reinterpret_cast<float4 *>(trow[h2] + lds_pos(base[u] + 4 * h)) =
                  make_float4(y[4 * h], y[4 * h + 1], y[4 * h + 2], y[4 * h + 3]);
          } else {
#pragma unroll
            for (int j = 0; j < B; ++j) trow[h2][lds_pos(base[u] + j * S)] = y[j];
          }
        }
      }
    }
  }
}

// Passes prog.pass[p0 .. p0+np), np >= 2, are single stages of radix B with strides that are
// powers of B inside the chunk, ascending (TRN false: the first stage has stride 1) or
// descending (TRN: the last one has).  blockDim.x * BPT = chunk / B blocks per stage and row.
// Q8: the blocks are rebuilt from the passes' int8 images instead of being read (BPT == 1).
template <typename TI, typename TO, int B, int BPT, bool TRN, bool Q8 = false>
__global__ __launch_bounds__(512) void harp_radix_kernel(const TI *__restrict__ X, int64_t ldx,
                                                         TO *__restrict__ Y, int64_t ldy,
                                                         int64_t n, int R, int nchunk, int chunk,
                                                         const Program *__restrict__ progp, int p0,
                                                         int np) {
  extern __shared__ float tile[];
  constexpr int V = B * B;
  using In = BlockIo<TI, B>;
  const int tid = threadIdx.x, NT = blockDim.x;
  const int kch = (int)(blockIdx.x % (unsigned)nchunk);
  const int64_t row0 = (int64_t)(blockIdx.x / (unsigned)nchunk) * R;
  const int nr = (int)((n - row0 < R) ? (n - row0) : R);
  const int dpad = lds_pos(chunk);
  const int nqc = chunk / B;   // blocks per stage in one chunk
  const Program &prog = *progp;
  const TI *Xt = X + row0 * ldx + (int64_t)kch * chunk;
  TO *Yt = Y + row0 * ldy + (int64_t)kch * chunk;

  float cur[BPT][V], nxt[BPT][V];
  // 16-byte loads from the four-values-per-load copy of the block parameters (pd.aux)
  typedef float vec4f __attribute__((ext_vector_type(4)));
  typedef const __attribute__((address_space(1))) vec4f *gfloat4_t;
  auto load_params = [&](const PassDesc &pd, float (&dst)[BPT][V]) {
    const gfloat4_t params = (gfloat4_t)pd.aux;
    const unsigned nq = (unsigned)pd.nq;
#pragma unroll
    for (int u = 0; u < BPT; ++u) {
      const unsigned qg = (unsigned)kch * nqc + tid + u * NT;
#pragma unroll
      for (int v4 = 0; v4 < V / 4; ++v4) {
        const vec4f f = params[(unsigned)v4 * nq + qg];
        dst[u][4 * v4] = f.x; dst[u][4 * v4 + 1] = f.y; dst[u][4 * v4 + 2] = f.z; dst[u][4 * v4 + 3] = f.w;
      }
    }
  };

  // first stage: every row of the tile is requested before the parameters are waited for
  const int S0 = prog.pass[p0].S;
  uint32_t raw[kRMax][BPT][B];
#pragma unroll
  for (int u = 0; u < BPT; ++u) {
    const int q = tid + u * NT, hi = q / S0, lo = q - hi * S0;
    const int base0 = hi * B * S0 + lo;
#pragma unroll
    for (int r = 0; r < kRMax; ++r) {
#pragma unroll
      for (int m = 0; m < B; ++m) raw[r][u][m] = 0u;
      if (r < nr) In::template load<!TRN>(Xt + (int64_t)r * ldx + base0, S0, raw[r][u]);
    }
  }
  if constexpr (Q8) {
    // codes of the next stage in flight while this stage's block is rebuilt and applied
    const unsigned qg = (unsigned)kch * nqc + tid;
    Q8Raw<B> rc, rn;
    q8_request<B>(prog.pass[p0], qg, rc);
    q8_request<B>(prog.pass[p0 + 1], qg, rn);
    q8_rebuild<B, TRN>(rc, prog.pass[p0].q8_flags, cur[0]);
    radix_pass<TI, TO, B, BPT, 0, !TRN>(tile, dpad, nr, S0, tid, NT, nqc, cur, raw, Yt, ldy);
    __syncthreads();
    for (int p = 1; p < np - 1; ++p) {
      rc = rn;
      q8_request<B>(prog.pass[p0 + p + 1], qg, rn);
      q8_rebuild<B, TRN>(rc, prog.pass[p0 + p].q8_flags, cur[0]);
      radix_pass<TI, TO, B, BPT, 1, false>(tile, dpad, nr, prog.pass[p0 + p].S, tid, NT, nqc, cur,
                                           raw, Yt, ldy);
      __syncthreads();
    }
    q8_rebuild<B, TRN>(rn, prog.pass[p0 + np - 1].q8_flags, cur[0]);
    radix_pass<TI, TO, B, BPT, 2, TRN>(tile, dpad, nr, prog.pass[p0 + np - 1].S, tid, NT, nqc, cur,
                                       raw, Yt, ldy);
    return;
  }
  load_params(prog.pass[p0], cur);
  load_params(prog.pass[p0 + 1], nxt);     // in flight during the first stage
  radix_pass<TI, TO, B, BPT, 0, !TRN>(tile, dpad, nr, S0, tid, NT, nqc, cur, raw, Yt, ldy);
  __syncthreads();
  for (int p = 1; p < np - 1; ++p) {
#pragma unroll
    for (int u = 0; u < BPT; ++u)
#pragma unroll
      for (int v = 0; v < V; ++v) cur[u][v] = nxt[u][v];
    load_params(prog.pass[p0 + p + 1], nxt);
    radix_pass<TI, TO, B, BPT, 1, false>(tile, dpad, nr, prog.pass[p0 + p].S, tid, NT, nqc, cur, raw,
                                         Yt, ldy);
    __syncthreads();
  }
  radix_pass<TI, TO, B, BPT, 2, TRN>(tile, dpad, nr, prog.pass[p0 + np - 1].S, tid, NT, nqc, nxt, raw,
                                     Yt, ldy);
}

// ------------------------------------------------------------------------------------------
// The same organisation for chunks whose stages have different radices in 3..8 (the greedy
// schedules of the paper: (8,8,8,7) inside d = 14336, (8,8,8,5) inside 5120): the radix of a
// stage is a run-time value dispatched to the compile-time bodies above, one block per thread
// (blockDim.x = the largest number of blocks of any stage; threads beyond a stage's count idle).
typedef float vec4f_t __attribute__((ext_vector_type(4)));

template <int B>
__device__ __forceinline__ void mixed_load_params(const PassDesc &pd, unsigned qg, bool active,
                                                  float (&dst)[64]) {
  if (!active) return;
  const unsigned nq = (unsigned)pd.nq;
  if (B == 4 || B == 8) {   // 16-byte loads from the four-values-per-load copy
    const __attribute__((address_space(1))) vec4f_t *p4 =
        (const __attribute__((address_space(1))) vec4f_t *)pd.aux;
#pragma unroll
    for (int v4 = 0; v4 < B * B / 4; ++v4) {
      const vec4f_t f = p4[(unsigned)v4 * nq + qg];
      dst[4 * v4] = f.x; dst[4 * v4 + 1] = f.y; dst[4 * v4 + 2] = f.z; dst[4 * v4 + 3] = f.w;
    }
  } else {
    const gfloat_t p1 = (gfloat_t)pd.params;
#pragma unroll
    for (int v = 0; v < B * B; ++v) dst[v] = p1[(unsigned)v * nq + qg];
  }
}

template <typename TI, typename TO, int B, int MODE, bool CONTIG>
__device__ __forceinline__ void mixed_pass(float *tile, int dpad, int nr, int S, int tid, int NT,
                                           int nqa, const float (&prm)[64], const TI *Xt,
                                           int64_t ldx, TO *Yt, int64_t ldy) {
  using In = BlockIo<TI, B>;
  uint32_t raw[kRMax][1][B];
  if (MODE == 0) {
    const int hi = tid / S, lo = tid - hi * S;
    const int base0 = hi * B * S + lo;
#pragma unroll
    for (int r = 0; r < kRMax; ++r) {
#pragma unroll
      for (int m = 0; m < B; ++m) raw[r][0][m] = 0u;
      if (r < nr && tid < nqa) In::template load<CONTIG>(Xt + (int64_t)r * ldx + base0, S, raw[r][0]);
    }
  }
  radix_pass<TI, TO, B, 1, MODE, CONTIG, true>(tile, dpad, nr, S, tid, NT, nqa,
                                         reinterpret_cast<const float(&)[1][B * B]>(prm), raw, Yt,
                                         ldy);
}

#define HARP_RADIX_SWITCH(b, STMT)                                        \
  switch (b) {                                                             \
    case 3: { constexpr int RB = 3; STMT; } break;                         \
    case 4: { constexpr int RB = 4; STMT; } break;                         \
    case 5: { constexpr int RB = 5; STMT; } break;                         \
    case 6: { constexpr int RB = 6; STMT; } break;                         \
    case 7: { constexpr int RB = 7; STMT; } break;                         \
    default: { constexpr int RB = 8; STMT; } break;                        \
  }

template <typename TI, typename TO>
__global__ __launch_bounds__(512) void harp_mixed_radix_kernel(
    const TI *__restrict__ X, int64_t ldx, TO *__restrict__ Y, int64_t ldy, int64_t n, int R,
    int nchunk, int chunk, const Program *__restrict__ progp, int p0, int np) {
  extern __shared__ float tile[];
  const int tid = threadIdx.x, NT = blockDim.x;
  const int kch = (int)(blockIdx.x % (unsigned)nchunk);
  const int64_t row0 = (int64_t)(blockIdx.x / (unsigned)nchunk) * R;
  const int nr = (int)((n - row0 < R) ? (n - row0) : R);
  const int dpad = lds_pos(chunk);
  const Program &prog = *progp;
  const TI *Xt = X + row0 * ldx + (int64_t)kch * chunk;
  TO *Yt = Y + row0 * ldy + (int64_t)kch * chunk;

  float cur[64], nxt[64];
  auto load_any = [&](const PassDesc &pd, float (&dst)[64]) {
    const int nqa = chunk / pd.b;
    const unsigned qg = (unsigned)kch * nqa + tid;
    HARP_RADIX_SWITCH(pd.b, mixed_load_params<RB>(pd, qg, tid < nqa, dst));
  };
  const PassDesc &first = prog.pass[p0];
  const PassDesc &last = prog.pass[p0 + np - 1];
  load_any(first, cur);
  load_any(prog.pass[p0 + 1], nxt);
  {
    const int nqa = chunk / first.b;
    if (first.S == 1 && first.b == 8)
      mixed_pass<TI, TO, 8, 0, true>(tile, dpad, nr, 1, tid, NT, nqa, cur, Xt, ldx, Yt, ldy);
    else if (first.S == 1 && first.b == 4)
      mixed_pass<TI, TO, 4, 0, true>(tile, dpad, nr, 1, tid, NT, nqa, cur, Xt, ldx, Yt, ldy);
    else
      HARP_RADIX_SWITCH(first.b, (mixed_pass<TI, TO, RB, 0, false>(tile, dpad, nr, first.S, tid, NT,
                                                                    nqa, cur, Xt, ldx, Yt, ldy)));
  }
  __syncthreads();
  for (int p = 1; p < np - 1; ++p) {
#pragma unroll
    for (int v = 0; v < 64; ++v) cur[v] = nxt[v];
    load_any(prog.pass[p0 + p + 1], nxt);
    const PassDesc &pd = prog.pass[p0 + p];
    const int nqa = chunk / pd.b;
    HARP_RADIX_SWITCH(pd.b, (mixed_pass<TI, TO, RB, 1, false>(tile, dpad, nr, pd.S, tid, NT, nqa, cur,
                                                              Xt, ldx, Yt, ldy)));
    __syncthreads();
  }
  {
    const int nqa = chunk / last.b;
    if (last.S == 1 && last.b == 8)
      mixed_pass<TI, TO, 8, 2, true>(tile, dpad, nr, 1, tid, NT, nqa, nxt, Xt, ldx, Yt, ldy);
    else if (last.S == 1 && last.b == 4)
      mixed_pass<TI, TO, 4, 2, true>(tile, dpad, nr, 1, tid, NT, nqa, nxt, Xt, ldx, Yt, ldy);
    else
      HARP_RADIX_SWITCH(last.b, (mixed_pass<TI, TO, RB, 2, false>(tile, dpad, nr, last.S, tid, NT, nqa,
                                                                  nxt, Xt, ldx, Yt, ldy)));
  }
}
#undef HARP_RADIX_SWITCH

// stages of radices 3..8, not all equal, that tile the chunk; returns the workgroup size or 0
int mixed_decode(const Program &pg, int p0, int np, int chunk) {
  if (np < 2 || np > 8) return 0;
  const PassDesc *ps = pg.pass + p0;
  int64_t prod = 1;
  int maxq = 0;
  for (int p = 0; p < np; ++p) {
    const int b = ps[p].b;
    if (ps[p].kind != PASS_SMALL || b < 3 || b > 8) return 0;
    if ((b == 4 || b == 8) && ps[p].aux == nullptr) return 0;
    if (chunk % b || ps[p].S < 1 || (chunk / b) % ps[p].S) return 0;
    prod *= b;
    maxq = std::max(maxq, chunk / b);
  }
  if (prod != chunk || maxq > 512) return 0;
  return (maxq + 63) / 64 * 64;
}

template <typename TI, typename TO>
harp_status_t launch_mixed_io(const harp_plan *plan, const HostProgram &hp, int p0, int np,
                              int chunk, int nt, const void *X, int64_t ldx, void *Y, int64_t ldy,
                              int64_t n, hipStream_t stream) {
  const int dpad = chunk + (chunk >> 6) * 8;
  int R = kRMax;
  while (R > 1 && (size_t)R * dpad * 4 > (size_t)plan->lds_bytes) --R;
  if ((size_t)R * dpad * 4 > (size_t)plan->lds_bytes) return HARP_ERR_UNSUPPORTED;
  if (plan->rows_override > 0 && plan->rows_override < R) R = plan->rows_override;
  if (R > n) R = (int)n;
  const int nchunk = (int)(plan->d / chunk);
  const int64_t tiles = ((n + R - 1) / R) * nchunk;
  if (tiles > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  const size_t lds = (size_t)R * dpad * 4;
  auto kern = harp_mixed_radix_kernel<TI, TO>;
  static thread_local int attr_done_dev = -1;   // per instantiation
  if (attr_done_dev != plan->device) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            plan->lds_bytes) != hipSuccess) {
      (void)hipGetLastError();
      return HARP_ERR_DEVICE;
    }
    attr_done_dev = plan->device;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(nt), lds, stream, (const TI *)X, ldx,
                     (TO *)Y, ldy, n, R, nchunk, chunk, hp.dev, p0, np);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

struct RadixShape {
  int B, np, nt, bpt;
  bool trn, ok;
  bool q8 = false;   // every pass carries an int8 image: the reconstructing variant can run
};

RadixShape radix_decode(const Program &pg, int p0, int np, int chunk) {
  RadixShape rs{0, np, 0, 0, false, false};
  if (np < 2 || np > 6) return rs;
  const PassDesc *ps = pg.pass + p0;
  const int B = ps[0].b;
  if (B != 4 && B != 8) return rs;
  int64_t prod = 1;
  for (int p = 0; p < np; ++p) {
    if (ps[p].kind != PASS_SMALL || ps[p].b != B || ps[p].aux == nullptr) return rs;
    prod *= B;
  }
  if (prod != chunk) return rs;
  // strides: the powers of B below the chunk, ascending or descending
  rs.trn = ps[0].S != 1;
  int64_t s = 1;
  for (int p = 0; p < np; ++p) {
    if (ps[rs.trn ? np - 1 - p : p].S != s) return rs;
    s *= B;
  }
  const int nqc = chunk / B;
  int nt = nqc < 512 ? nqc : 512;
  if (nt < 64 || nqc % nt) return rs;
  const int bpt = nqc / nt;
  if (bpt != 1 && bpt != 2) return rs;
  if (B == 8 && bpt != 1) return rs;
  rs.B = B;
  rs.nt = nt;
  rs.bpt = bpt;
  rs.ok = true;
  rs.q8 = (bpt == 1);
  for (int p = 0; p < np; ++p) rs.q8 = rs.q8 && ps[p].q8 != nullptr;
  return rs;
}

template <typename TI, typename TO, int B, int BPT, bool TRN, bool Q8 = false>
harp_status_t launch_radix_inst(const harp_plan *plan, const HostProgram &hp, int p0, int np,
                                int chunk, int nt, const void *X, int64_t ldx, void *Y,
                                int64_t ldy, int64_t n, hipStream_t stream) {
  const int dpad = chunk + (chunk >> 6) * 8;
  int R = kRMax;
  while (R > 1 && (size_t)R * dpad * 4 > (size_t)plan->lds_bytes) --R;
  if ((size_t)R * dpad * 4 > (size_t)plan->lds_bytes) return HARP_ERR_UNSUPPORTED;
  if (plan->rows_override > 0 && plan->rows_override < R) R = plan->rows_override;
  if (R > n) R = (int)n;
  const int nchunk = (int)(plan->d / chunk);
  const int64_t tiles = ((n + R - 1) / R) * nchunk;
  if (tiles > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  const size_t lds = (size_t)R * dpad * 4;
  auto kern = harp_radix_kernel<TI, TO, B, BPT, TRN, Q8>;
  static thread_local int attr_done_dev = -1;   // per instantiation
  if (attr_done_dev != plan->device) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            plan->lds_bytes) != hipSuccess) {
      (void)hipGetLastError();
      return HARP_ERR_DEVICE;
    }
    attr_done_dev = plan->device;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(nt), lds, stream, (const TI *)X, ldx,
                     (TO *)Y, ldy, n, R, nchunk, chunk, hp.dev, p0, np);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

template <typename TI, typename TO>
harp_status_t launch_radix_io(const harp_plan *plan, const HostProgram &hp, int p0,
                              const RadixShape &rs, int chunk, const void *X, int64_t ldx, void *Y,
                              int64_t ldy, int64_t n, hipStream_t stream) {
#define HARP_RADIX_CASE(B_, BPT_)                                                              \
  (rs.trn ? launch_radix_inst<TI, TO, B_, BPT_, true>(plan, hp, p0, rs.np, chunk, rs.nt, X, ldx, \
                                                      Y, ldy, n, stream)                         \
          : launch_radix_inst<TI, TO, B_, BPT_, false>(plan, hp, p0, rs.np, chunk, rs.nt, X,     \
                                                       ldx, Y, ldy, n, stream))
#define HARP_RADIX_CASE_Q8(B_)                                                                     \
  (rs.trn ? launch_radix_inst<TI, TO, B_, 1, true, true>(plan, hp, p0, rs.np, chunk, rs.nt, X, ldx, \
                                                         Y, ldy, n, stream)                         \
          : launch_radix_inst<TI, TO, B_, 1, false, true>(plan, hp, p0, rs.np, chunk, rs.nt, X,     \
                                                          ldx, Y, ldy, n, stream))
  if (rs.q8 && plan->theta_in_kernel) {
    if (rs.B == 8) return HARP_RADIX_CASE_Q8(8);
    return HARP_RADIX_CASE_Q8(4);
  }
#undef HARP_RADIX_CASE_Q8
  if (rs.B == 8) return HARP_RADIX_CASE(8, 1);
  if (rs.bpt == 1) return HARP_RADIX_CASE(4, 1);
  return HARP_RADIX_CASE(4, 2);
#undef HARP_RADIX_CASE
}

}  // namespace

bool radix_supported(const harp_plan *plan, const Program &pg, int p0, int np, int chunk,
                     const void *X, int64_t ldx, const void *Y, int64_t ldy) {
  if (plan->algo == HARP_ALGO_GENERIC) return false;
  if (!radix_decode(pg, p0, np, chunk).ok && mixed_decode(pg, p0, np, chunk) == 0) return false;
  // 16-byte accesses of the contiguous stage for either element type
  if ((ldx % 8) || (ldy % 8) || ((uintptr_t)X % 16) || ((uintptr_t)Y % 16)) return false;
  return (size_t)(chunk + (chunk >> 6) * 8) * 4 <= (size_t)plan->lds_bytes;
}

// true when launch_radix_kernel would take the variant that rebuilds the blocks from int8 codes
bool radix_rebuilds_in_kernel(const harp_plan *plan, const Program &pg, int p0, int np, int chunk) {
  return plan->theta_in_kernel && radix_decode(pg, p0, np, chunk).q8;
}

harp_status_t launch_radix_kernel(const harp_plan *plan, const HostProgram &hp, int p0, int np,
                                  int chunk, const void *X, int64_t ldx, harp_dtype_t dt_in,
                                  void *Y, int64_t ldy, harp_dtype_t dt_out, int64_t n,
                                  hipStream_t stream) {
  const RadixShape rs = radix_decode(hp.prog, p0, np, chunk);
  if (!rs.ok) {
    const int nt = mixed_decode(hp.prog, p0, np, chunk);
    if (nt == 0) return HARP_ERR_UNSUPPORTED;
    if (dt_in == HARP_BF16 && dt_out == HARP_BF16)
      return launch_mixed_io<uint16_t, uint16_t>(plan, hp, p0, np, chunk, nt, X, ldx, Y, ldy, n, stream);
    if (dt_in == HARP_BF16 && dt_out == HARP_F32)
      return launch_mixed_io<uint16_t, float>(plan, hp, p0, np, chunk, nt, X, ldx, Y, ldy, n, stream);
    if (dt_in == HARP_F32 && dt_out == HARP_BF16)
      return launch_mixed_io<float, uint16_t>(plan, hp, p0, np, chunk, nt, X, ldx, Y, ldy, n, stream);
    return launch_mixed_io<float, float>(plan, hp, p0, np, chunk, nt, X, ldx, Y, ldy, n, stream);
  }
  if (dt_in == HARP_BF16 && dt_out == HARP_BF16)
    return launch_radix_io<uint16_t, uint16_t>(plan, hp, p0, rs, chunk, X, ldx, Y, ldy, n, stream);
  if (dt_in == HARP_BF16 && dt_out == HARP_F32)
    return launch_radix_io<uint16_t, float>(plan, hp, p0, rs, chunk, X, ldx, Y, ldy, n, stream);
  if (dt_in == HARP_F32 && dt_out == HARP_BF16)
    return launch_radix_io<float, uint16_t>(plan, hp, p0, rs, chunk, X, ldx, Y, ldy, n, stream);
  return launch_radix_io<float, float>(plan, hp, p0, rs, chunk, X, ldx, Y, ldy, n, stream);
}

}  // namespace harp
