// HIP kernels for gfx950 and their launchers.
//
// harp_tile_kernel: one workgroup owns a tile of R rows.  The tile is loaded once from
// device memory into LDS as float32 (bf16 widened), every stage of the processor is executed
// on that on-chip copy, and the tile is written back once (one round-to-nearest-even to
// bf16).  Between the load and the store nothing touches device memory except the stream of
// stage parameters.  The processor's +-1 signs never appear here: the plan folds them into
// the stage parameters.
//
// The stages are grouped into passes (see PassDesc).  Within a pass a thread owns one
// sub-tensor position q of the row for several rows of the tile: it reads the parameters
// of its 2x2 / bxb blocks into registers once and reuses them for every row it handles,
// so the parameter stream is read once per tile, not once per row (Alg. 1's K_t[c] does not
// depend on the row).  The stride permutation P_t of Eq. (7) is never materialised: a
// stage's coordinates alpha*b*s + r*s + beta are addressed directly in LDS (Lemma 1).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <stdlib.h>

#include <algorithm>

#include "harp_internal.h"

namespace harp {

namespace {

// ------------------------------------------------------------------------------------------
// element conversion
__device__ __forceinline__ float widen_bf16(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  // hardware round-to-nearest-even conversion (v_cvt_pk_bf16_f32 on gfx950)
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  bf2 v;
  v.x = (__bf16)lo;
  v.y = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ uint16_t narrow_bf16(float f) {
  __bf16 h = (__bf16)f;
  return __builtin_bit_cast(uint16_t, h);
}

template <typename T>
struct IoTraits;
template <>
struct IoTraits<float> {
  static constexpr int kVec = 4;  // elements per 16-byte access
};
template <>
struct IoTraits<uint16_t> {
  static constexpr int kVec = 8;
};

__device__ __forceinline__ void load_vec(const float *p, float (&v)[4]) {
  const float4 t = *reinterpret_cast<const float4 *>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ __forceinline__ void load_vec(const uint16_t *p, float (&v)[8]) {
  const uint4 t = *reinterpret_cast<const uint4 *>(p);
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
  v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xffff0000u);
  v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xffff0000u);
}
__device__ __forceinline__ void store_vec(float *p, const float (&v)[4]) {
  *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store_vec(uint16_t *p, const float (&v)[8]) {
  uint4 t;
  t.x = pack_bf16x2(v[0], v[1]);
  t.y = pack_bf16x2(v[2], v[3]);
  t.z = pack_bf16x2(v[4], v[5]);
  t.w = pack_bf16x2(v[6], v[7]);
  *reinterpret_cast<uint4 *>(p) = t;
}
__device__ __forceinline__ float load_one(const float *p) { return *p; }
__device__ __forceinline__ float load_one(const uint16_t *p) { return widen_bf16(*p); }
__device__ __forceinline__ void store_one(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_one(uint16_t *p, float v) { *p = narrow_bf16(v); }

// ------------------------------------------------------------------------------------------
// passes (all operate on the float32 LDS tile, row stride d)

// K consecutive radix-2 stages on sub-tensors of P = 2^K coordinates.
// FORM 0: dense 2x2 blocks, 4 values per pair.  FORM 1: orthogonal blocks as three lifting
// steps, 2 values (a, b) per pair: x0 += a x1; x1 += b x0; x0 += a x1.  FORM 2: as FORM 1
// but the K-th stage is dense (its 4-value pairs follow the (K-1) * P lifted values).
// FORM 3 / 4: as FORM 1 / 2 with two shears per pair instead of three lifting steps:
// (x0, x1) <- (x0 + a x1, x1 + b x0), output scales deferred by the plan.
template <int K, bool DESC, int FORM>
__device__ __forceinline__ void pass_pow2(float *tile, int d, int nr, const PassDesc &pd, int kch,
                                          int tid, int nt) {
  constexpr int P = 1 << K;
  constexpr int NV = (FORM == 0) ? K * (P / 2) * 4 : ((FORM == 1 || FORM == 3) ? K * P : (K + 1) * P);
  // the tile rows are chunk `kch` (d coordinates) of the full rows: nq sub-tensors here,
  // numbered qoff .. qoff + nq - 1 among the pd.nq sub-tensors of a full row
  const int nq = d / P, S = pd.S, nqg = pd.nq, qoff = kch * nq;
  const float *__restrict__ params = pd.params;
  int RG = 1;
  if (nq < nt) {
    RG = nt / nq;
    if (RG > nr) RG = nr;
  }
  const int items = nq * RG;
  for (int it = tid; it < items; it += nt) {
    int q = it, rg = 0;
    if (RG > 1) {
      rg = it / nq;
      q = it - rg * nq;
    }
    float prm[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) prm[v] = params[(size_t)v * nqg + qoff + q];
    const int hi = q / S, lo = q - hi * S;
    float *tb = tile + hi * P * S + lo;
    for (int row = rg; row < nr; row += RG) {
      float *t = tb + row * d;
      float x[P];
#pragma unroll
      for (int j = 0; j < P; ++j) x[j] = t[j * S];
#pragma unroll
      for (int e = 0; e < K; ++e) {
        const int bp = DESC ? K - 1 - e : e;
        const bool dense = (FORM == 0) || ((FORM == 2 || FORM == 4) && e == K - 1);
#pragma unroll
        for (int p = 0; p < P / 2; ++p) {
          const int j0 = ((p >> bp) << (bp + 1)) | (p & ((1 << bp) - 1));
          const int j1 = j0 | (1 << bp);
          float x0 = x[j0], x1 = x[j1];
          if (!dense) {
            const float a = prm[(e * (P / 2) + p) * 2 + 0], b = prm[(e * (P / 2) + p) * 2 + 1];
            if (FORM >= 3) {
              x[j0] = fmaf(a, x1, x0);
              x[j1] = fmaf(b, x0, x1);
            } else {
              x0 = fmaf(a, x1, x0);
              x1 = fmaf(b, x0, x1);
              x0 = fmaf(a, x1, x0);
              x[j0] = x0;
              x[j1] = x1;
            }
          } else {
            const int v0 = (FORM == 0) ? (e * (P / 2) + p) * 4 : (K - 1) * P + p * 4;
            const float k00 = prm[v0 + 0], k01 = prm[v0 + 1], k10 = prm[v0 + 2], k11 = prm[v0 + 3];
            x[j0] = fmaf(x1, k10, x0 * k00);
            x[j1] = fmaf(x1, k11, x0 * k01);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < P; ++j) t[j * S] = x[j];
    }
  }
}

// One stage of compile-time radix B (3..8): the whole block lives in registers.
template <int B>
__device__ __forceinline__ void pass_small(float *tile, int d, int nr, const PassDesc &pd, int kch,
                                           int tid, int nt) {
  const int nq = d / B, S = pd.S, nqg = pd.nq, qoff = kch * nq;
  const float *__restrict__ params = pd.params;
  int RG = 1;
  if (nq < nt) {
    RG = nt / nq;
    if (RG > nr) RG = nr;
  }
  const int items = nq * RG;
  for (int it = tid; it < items; it += nt) {
    int q = it, rg = 0;
    if (RG > 1) {
      rg = it / nq;
      q = it - rg * nq;
    }
    float prm[B * B];
#pragma unroll
    for (int v = 0; v < B * B; ++v) prm[v] = params[(size_t)v * nqg + qoff + q];
    const int hi = q / S, lo = q - hi * S;
    float *tb = tile + hi * B * S + lo;
    for (int row = rg; row < nr; row += RG) {
      float *t = tb + row * d;
      float x[B], y[B];
#pragma unroll
      for (int r = 0; r < B; ++r) x[r] = t[r * S];
#pragma unroll
      for (int r2 = 0; r2 < B; ++r2) {
        float acc = x[0] * prm[r2];
#pragma unroll
        for (int r = 1; r < B; ++r) acc = fmaf(x[r], prm[r * B + r2], acc);
        y[r2] = acc;
      }
#pragma unroll
      for (int r = 0; r < B; ++r) t[r * S] = y[r];
    }
  }
}

// One stage of run-time radix b <= BMAX: a thread owns one block of one row; the block's
// coordinates are held in registers, the b*b parameters are streamed.
template <int BMAX>
__device__ __forceinline__ void pass_generic(float *tile, int d, int nr, const PassDesc &pd,
                                             int kch, int tid, int nt) {
  const int S = pd.S, b = pd.b, nq = d / b, nqg = pd.nq, qoff = kch * nq;
  const float *__restrict__ params = pd.params;
  const int items = nq * nr;
  for (int it = tid; it < items; it += nt) {
    const int row = it / nq, q = it - row * nq;
    const int hi = q / S, lo = q - hi * S;
    float *t = tile + row * d + hi * b * S + lo;
    float x[BMAX];
#pragma unroll
    for (int r = 0; r < BMAX; ++r) x[r] = (r < b) ? t[r * S] : 0.0f;
    for (int r2 = 0; r2 < b; ++r2) {
      const float *pp = params + (size_t)r2 * nqg + qoff + q;
      float acc = 0.0f;
#pragma unroll
      for (int r = 0; r < BMAX; ++r)   // unconditional loads (x[r] is zero past the radix): all in flight
        acc = fmaf(x[r], pp[(size_t)(r < b ? r : b - 1) * b * nqg], acc);
      t[r2 * S] = acc;
    }
  }
}

template <bool DESC, int FORM>
__device__ __forceinline__ void dispatch_pow2(float *tile, int d, int nr, const PassDesc &pd,
                                              int kch, int tid, int nt) {
  switch (pd.k) {
    case 1: pass_pow2<1, DESC, FORM>(tile, d, nr, pd, kch, tid, nt); break;
    case 2: pass_pow2<2, DESC, FORM>(tile, d, nr, pd, kch, tid, nt); break;
    case 3: pass_pow2<3, DESC, FORM>(tile, d, nr, pd, kch, tid, nt); break;
    case 4:
      if (FORM != 0) pass_pow2<4, DESC, (FORM == 0 ? 1 : FORM)>(tile, d, nr, pd, kch, tid, nt);
      break;
    default: break;
  }
}

__device__ __forceinline__ void run_pass(float *tile, int d, int nr, const PassDesc &pd, int kch,
                                         int tid, int nt) {
  switch (pd.kind) {
    case PASS_POW2_DENSE:
      if (pd.desc) dispatch_pow2<true, 0>(tile, d, nr, pd, kch, tid, nt);
      else dispatch_pow2<false, 0>(tile, d, nr, pd, kch, tid, nt);
      break;
    case PASS_POW2_LIFT:
      if (pd.desc) dispatch_pow2<true, 1>(tile, d, nr, pd, kch, tid, nt);
      else dispatch_pow2<false, 1>(tile, d, nr, pd, kch, tid, nt);
      break;
    case PASS_POW2_LIFT_LD:
      if (pd.desc) dispatch_pow2<true, 2>(tile, d, nr, pd, kch, tid, nt);
      else dispatch_pow2<false, 2>(tile, d, nr, pd, kch, tid, nt);
      break;
    case PASS_POW2_SCALED:
      if (pd.desc) dispatch_pow2<true, 3>(tile, d, nr, pd, kch, tid, nt);
      else dispatch_pow2<false, 3>(tile, d, nr, pd, kch, tid, nt);
      break;
    case PASS_POW2_SCALED_LD:
      if (pd.desc) dispatch_pow2<true, 4>(tile, d, nr, pd, kch, tid, nt);
      else dispatch_pow2<false, 4>(tile, d, nr, pd, kch, tid, nt);
      break;
    case PASS_SMALL:
      switch (pd.b) {
        case 3: pass_small<3>(tile, d, nr, pd, kch, tid, nt); break;
        case 4: pass_small<4>(tile, d, nr, pd, kch, tid, nt); break;
        case 5: pass_small<5>(tile, d, nr, pd, kch, tid, nt); break;
        case 6: pass_small<6>(tile, d, nr, pd, kch, tid, nt); break;
        case 7: pass_small<7>(tile, d, nr, pd, kch, tid, nt); break;
        case 8: pass_small<8>(tile, d, nr, pd, kch, tid, nt); break;
        default: break;
      }
      break;
    default:
      if (pd.b <= 8) pass_generic<8>(tile, d, nr, pd, kch, tid, nt);
      else if (pd.b <= 16) pass_generic<16>(tile, d, nr, pd, kch, tid, nt);
      else if (pd.b <= 32) pass_generic<32>(tile, d, nr, pd, kch, tid, nt);
      else if (pd.b <= 48) pass_generic<48>(tile, d, nr, pd, kch, tid, nt);
      else pass_generic<64>(tile, d, nr, pd, kch, tid, nt);
      break;
  }
}

// ------------------------------------------------------------------------------------------
template <typename TI, typename TO>
__global__ __launch_bounds__(512) void harp_tile_kernel(const TI *__restrict__ X, int64_t ldx,
                                                         TO *__restrict__ Y, int64_t ldy, int64_t n,
                                                         int d, int nchunk, int R, int vec_in,
                                                         int vec_out,
                                                         const Program *__restrict__ progp, int p0,
                                                         int p1) {
  // d = coordinates of the on-chip chunk; a row has nchunk of them (1: the whole row).
  // Workgroup -> (chunk kch, tile of R rows); passes p0 .. p1-1 are local to a chunk.
  extern __shared__ float tile[];
  const int tid = threadIdx.x, nt = blockDim.x;
  const int kch = (int)(blockIdx.x % (unsigned)nchunk);
  const int64_t row0 = (int64_t)(blockIdx.x / (unsigned)nchunk) * R;
  const int nr = (int)((n - row0 < R) ? (n - row0) : R);
  const Program &prog = *progp;   // uniform address: fetched with scalar loads
  X += (int64_t)kch * d;
  Y += (int64_t)kch * d;

  // ---- load: device memory -> LDS (float32)
  if (vec_in) {
    constexpr int VI = IoTraits<TI>::kVec;
    const int cpr = d / VI;
    int row = 0, ch = tid;
    while (ch >= cpr) { ch -= cpr; ++row; }
    while (row < nr) {
      float v[VI];
      load_vec(X + (row0 + row) * ldx + (int64_t)ch * VI, v);
      float *t = tile + row * d + ch * VI;
#pragma unroll
      for (int k = 0; k < VI; k += 4)
        *reinterpret_cast<float4 *>(t + k) = make_float4(v[k], v[k + 1], v[k + 2], v[k + 3]);
      ch += nt;
      while (ch >= cpr) { ch -= cpr; ++row; }
    }
  } else {
    for (int row = 0; row < nr; ++row)
      for (int i = tid; i < d; i += nt) {
        tile[row * d + i] = load_one(X + (row0 + row) * ldx + i);
      }
  }
  __syncthreads();

  // ---- all stages on chip
  for (int p = p0; p < p1; ++p) {
    run_pass(tile, d, nr, prog.pass[p], kch, tid, nt);
    __syncthreads();
  }

  // ---- store: LDS -> device memory
  if (vec_out) {
    constexpr int VO = IoTraits<TO>::kVec;
    const int cpr = d / VO;
    int row = 0, ch = tid;
    while (ch >= cpr) { ch -= cpr; ++row; }
    while (row < nr) {
      float v[VO];
      const float *t = tile + row * d + ch * VO;
#pragma unroll
      for (int k = 0; k < VO; k += 4) {
        const float4 f = *reinterpret_cast<const float4 *>(t + k);
        v[k] = f.x; v[k + 1] = f.y; v[k + 2] = f.z; v[k + 3] = f.w;
      }
      store_vec(Y + (row0 + row) * ldy + (int64_t)ch * VO, v);
      ch += nt;
      while (ch >= cpr) { ch -= cpr; ++row; }
    }
  } else {
    for (int row = 0; row < nr; ++row)
      for (int i = tid; i < d; i += nt) {
        store_one(Y + (row0 + row) * ldy + i, tile[row * d + i]);
      }
  }
}

// ------------------------------------------------------------------------------------------
// One pass streamed through device memory: a thread owns sub-tensor q of the row (consecutive
// threads = consecutive q = consecutive addresses for every j), keeps the pass parameters in
// registers and walks down the rows of its row block.  Used for the passes on the digits above
// the on-chip chunk of a split program.  No LDS, no barrier.
template <int K, bool DESC, int FORM>
struct OpPow2 {
  static constexpr int P = 1 << K;
  static constexpr int NV = (FORM == 0) ? K * (P / 2) * 4 : ((FORM == 1 || FORM == 3) ? K * P : (K + 1) * P);
  __device__ static __forceinline__ void apply(float (&x)[P], const float (&prm)[NV]) {
#pragma unroll
    for (int e = 0; e < K; ++e) {
      const int bp = DESC ? K - 1 - e : e;
      const bool dense = (FORM == 0) || ((FORM == 2 || FORM == 4) && e == K - 1);
#pragma unroll
      for (int p = 0; p < P / 2; ++p) {
        const int j0 = ((p >> bp) << (bp + 1)) | (p & ((1 << bp) - 1));
        const int j1 = j0 | (1 << bp);
        float x0 = x[j0], x1 = x[j1];
        if (!dense) {
          const float a = prm[(e * (P / 2) + p) * 2 + 0], b = prm[(e * (P / 2) + p) * 2 + 1];
          if (FORM >= 3) {
            x[j0] = fmaf(a, x1, x0);
            x[j1] = fmaf(b, x0, x1);
          } else {
            x0 = fmaf(a, x1, x0);
            x1 = fmaf(b, x0, x1);
            x0 = fmaf(a, x1, x0);
            x[j0] = x0;
            x[j1] = x1;
          }
        } else {
          const int v0 = (FORM == 0) ? (e * (P / 2) + p) * 4 : (K - 1) * P + p * 4;
          x[j0] = fmaf(x1, prm[v0 + 2], x0 * prm[v0 + 0]);
          x[j1] = fmaf(x1, prm[v0 + 3], x0 * prm[v0 + 1]);
        }
      }
    }
  }
};

template <int B>
struct OpSmall {
  static constexpr int P = B;
  static constexpr int NV = B * B;
  __device__ static __forceinline__ void apply(float (&x)[P], const float (&prm)[NV]) {
    float y[B];
#pragma unroll
    for (int r2 = 0; r2 < B; ++r2) {
      float acc = x[0] * prm[r2];
#pragma unroll
      for (int r = 1; r < B; ++r) acc = fmaf(x[r], prm[r * B + r2], acc);
      y[r2] = acc;
    }
#pragma unroll
    for (int r = 0; r < B; ++r) x[r] = y[r];
  }
};

// K stages of radix B on adjacent digits of a sub-tensor of B^K coordinates (element j of the
// thread = digits (e_0 .. e_{K-1}) of j in base B, digit p at stride B^p), in execution order
// k = 0 .. K-1 on digit p = k (DESC: K-1-k).
template <int B, int K, bool DESC>
struct OpSmallChain {
  static constexpr int ipow(int b, int k) { return k == 0 ? 1 : b * ipow(b, k - 1); }
  static constexpr int P = ipow(B, K);
  static constexpr int NB = P / B;           // blocks per stage inside the sub-tensor
  static constexpr int NV = K * NB * B * B;
  __device__ static __forceinline__ void apply(float (&x)[P], const float (&prm)[NV]) {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int p = DESC ? K - 1 - k : k;
      const int sp = ipow(B, p);
#pragma unroll
      for (int o = 0; o < NB; ++o) {
        const int j0 = (o / sp) * sp * B + o % sp;   // digit p = 0, the others = o
        const float *kb = prm + (k * NB + o) * B * B;
        float y[B];
#pragma unroll
        for (int r2 = 0; r2 < B; ++r2) {
          float acc = x[j0] * kb[r2];
#pragma unroll
          for (int r = 1; r < B; ++r) acc = fmaf(x[j0 + r * sp], kb[r * B + r2], acc);
          y[r2] = acc;
        }
#pragma unroll
        for (int r = 0; r < B; ++r) x[j0 + r * sp] = y[r];
      }
    }
  }
};

__device__ __forceinline__ float stream_load(const void *p, int64_t i, int bf16) {
  return bf16 ? widen_bf16(static_cast<const uint16_t *>(p)[i]) : static_cast<const float *>(p)[i];
}
__device__ __forceinline__ void stream_store(void *p, int64_t i, int bf16, float v) {
  if (bf16) static_cast<uint16_t *>(p)[i] = narrow_bf16(v);
  else static_cast<float *>(p)[i] = v;
}

// element access of the streamed kernels, by element type
__device__ __forceinline__ float stream_widen(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float stream_widen(float v) { return v; }
__device__ __forceinline__ void stream_put(uint16_t *p, float v) { *p = narrow_bf16(v); }
__device__ __forceinline__ void stream_put(float *p, float v) { *p = v; }

// One thread per sub-tensor q, walking down its block of rows with the parameters in registers;
// two rows in flight (the loads of row + 1 are issued before row is computed and stored).
// Element types are template parameters and all offsets inside a row are 32-bit, so a row
// costs the arithmetic of the stage plus two pointer increments.
template <class OP, typename TI, typename TO>
__global__ __launch_bounds__(256) void harp_stream_kernel(const TI *__restrict__ X, int64_t ldx,
                                                          TO *__restrict__ Y, int64_t ldy,
                                                          int64_t n, int rows_per_block,
                                                          const float *__restrict__ params, int nq,
                                                          int S) {
  constexpr int P = OP::P, NV = OP::NV;
  const int q = blockIdx.x * 256 + threadIdx.x;
  if (q >= nq) return;
  float prm[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) prm[v] = params[(size_t)v * nq + q];
  const int hi = q / S, lo = q - hi * S;
  const int64_t base = (int64_t)hi * P * S + lo;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
  const int nr = (int)((r0 + rows_per_block < n) ? rows_per_block : n - r0);
  const TI *xp = X + r0 * ldx + base;
  TO *yp = Y + r0 * ldy + base;
  // Two rows in flight in two named buffers (a: even rows of the block, b: odd rows), each as
  // loaded (bf16 zero-extended to 32 bits, widened only when its turn comes).  Every load and
  // store is unconditional -- past the last row the pointers stop moving, so the last row is
  // loaded, computed and stored a second time with the same bits -- and the scheduling barriers
  // keep the order written here: a wait for a buffer then always follows the same 2 P younger
  // operations and is a wait for that buffer only, not for the stores issued since.
  typedef typename std::conditional<sizeof(TI) == 2, uint32_t, float>::type Raw;
  Raw a[P], b[P];
#pragma unroll
  for (int j = 0; j < P; ++j) a[j] = (Raw)xp[(unsigned)(j * S)];
  for (int r = 0; r < nr; r += 2) {
    const TI *xb = (r + 1 < nr) ? xp + ldx : xp;
    TO *yb = (r + 1 < nr) ? yp + ldy : yp;
#pragma unroll
    for (int j = 0; j < P; ++j) b[j] = (Raw)xb[(unsigned)(j * S)];
    __builtin_amdgcn_sched_barrier(0);
    {
      float x[P];
#pragma unroll
      for (int j = 0; j < P; ++j) x[j] = stream_widen(a[j]);
      OP::apply(x, prm);
#pragma unroll
      for (int j = 0; j < P; ++j) stream_put(yp + (unsigned)(j * S), x[j]);
    }
    __builtin_amdgcn_sched_barrier(0);
    xp = (r + 2 < nr) ? xb + ldx : xb;
#pragma unroll
    for (int j = 0; j < P; ++j) a[j] = (Raw)xp[(unsigned)(j * S)];
    __builtin_amdgcn_sched_barrier(0);
    {
      float x[P];
#pragma unroll
      for (int j = 0; j < P; ++j) x[j] = stream_widen(b[j]);
      OP::apply(x, prm);
#pragma unroll
      for (int j = 0; j < P; ++j) stream_put(yb + (unsigned)(j * S), x[j]);
    }
    __builtin_amdgcn_sched_barrier(0);
    yp = yb + ldy;
  }
}

// The same stage between a bf16 side and the block-scaled half intermediate (2 bytes per
// coordinate on both sides).  A thread owns TWO neighbouring sub-tensors (coordinates lo, lo + 1
// of every j: one 32-bit access per j and row), eight lanes share a segment of 16 coordinates
// and its exponent byte.  ZIN: halves in, bf16 out (the stage is the last of a forward
// program); otherwise bf16 in, halves out (the first of a transposed one): the segment's
// largest magnitude is found with three DPP steps (lane ^ 1, lane ^ 2, mirror of the eight).
// Two rows in flight as above; S and the sub-tensor count are even, S a multiple of 16.
template <class OP, bool ZIN>
__global__ __launch_bounds__(256) void harp_stream_z16_kernel(const uint16_t *__restrict__ X,
                                                              int64_t ldx, uint16_t *__restrict__ Y,
                                                              int64_t ldy, int64_t n,
                                                              int rows_per_block,
                                                              const float *__restrict__ params,
                                                              int nq, int S, int d) {
  constexpr int P = OP::P, NV = OP::NV;
  const int q = 2 * (blockIdx.x * 256 + threadIdx.x);
  if (q >= nq) return;
  float prm[2][NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    prm[0][v] = params[(size_t)v * nq + q];
    prm[1][v] = params[(size_t)v * nq + q + 1];
  }
  const int hi = q / S, lo = q - hi * S;
  const unsigned base = (unsigned)hi * P * S + lo;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
  const int nr = (int)((r0 + rows_per_block < n) ? rows_per_block : n - r0);
  const uint16_t *xp = X + r0 * ldx;
  uint16_t *yp = Y + r0 * ldy;
  struct Raw {
    uint32_t w[P];
    uint32_t e[ZIN ? P : 1];
  };
  auto request = [&](const uint16_t *xr, Raw &raw) {
#pragma unroll
    for (int j = 0; j < P; ++j) {
      raw.w[j] = *reinterpret_cast<const uint32_t *>(xr + base + (unsigned)(j * S));
      if (ZIN) raw.e[j] = reinterpret_cast<const uint8_t *>(xr + d)[(base + (unsigned)(j * S)) >> 4];
    }
  };
  auto finish = [&](const Raw &raw, uint16_t *yr) {
    float x0[P], x1[P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
      if (ZIN) {
        z16_unpack(raw.w[j], z16_up(raw.e[j]), x0[j], x1[j]);
      } else {
        x0[j] = __uint_as_float(raw.w[j] << 16);
        x1[j] = __uint_as_float(raw.w[j] & 0xffff0000u);
      }
    }
    OP::apply(x0, prm[0]);
    OP::apply(x1, prm[1]);
    if (ZIN) {
#pragma unroll
      for (int j = 0; j < P; ++j)
        *reinterpret_cast<uint32_t *>(yr + base + (unsigned)(j * S)) = pack_bf16x2(x0[j], x1[j]);
    } else {
      // largest magnitude of every segment: the P reductions run side by side (as bit patterns
      // of non-negative floats, which order like unsigned integers)
      uint32_t mx[P];
#pragma unroll
      for (int j = 0; j < P; ++j) mx[j] = __float_as_uint(fmaxf(fabsf(x0[j]), fabsf(x1[j])));
#pragma unroll
      for (int j = 0; j < P; ++j)
        mx[j] = max(mx[j], (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mx[j], 0xB1 /* quad_perm [1,0,3,2] */, 0xf, 0xf, false));
#pragma unroll
      for (int j = 0; j < P; ++j)
        mx[j] = max(mx[j], (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mx[j], 0x4E /* quad_perm [2,3,0,1] */, 0xf, 0xf, false));
#pragma unroll
      for (int j = 0; j < P; ++j)
        mx[j] = max(mx[j], (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mx[j], 0x141 /* row_half_mirror */, 0xf, 0xf, false));
#pragma unroll
      for (int j = 0; j < P; ++j) {
        uint32_t ex = mx[j] >> 23;
        ex = ex > 253u ? 253u : ex;
        mx[j] = ex;
        const float f = z16_down(ex);
        *reinterpret_cast<uint32_t *>(yr + base + (unsigned)(j * S)) = z16_pack(x0[j] * f, x1[j] * f);
      }
      if ((threadIdx.x & 7) == 0) {
#pragma unroll
        for (int j = 0; j < P; ++j)
          reinterpret_cast<uint8_t *>(yr + d)[(base + (unsigned)(j * S)) >> 4] = (uint8_t)mx[j];
      }
    }
  };
  Raw a, b;
  request(xp, a);
  for (int r = 0; r < nr; r += 2) {
    const uint16_t *xb = (r + 1 < nr) ? xp + ldx : xp;
    uint16_t *yb = (r + 1 < nr) ? yp + ldy : yp;
    request(xb, b);
    __builtin_amdgcn_sched_barrier(0);
    finish(a, yp);
    __builtin_amdgcn_sched_barrier(0);
    xp = (r + 2 < nr) ? xb + ldx : xb;
    request(xp, a);
    __builtin_amdgcn_sched_barrier(0);
    finish(b, yb);
    __builtin_amdgcn_sched_barrier(0);
    yp = yb + ldy;
  }
}

// The same stage with the rows staged through LDS, for strides that are multiples of 256: a
// workgroup owns a strip of 256 consecutive sub-tensors and walks down its rows in pairs.
// Device memory is touched with 16-byte accesses only (one piece of 8 coordinates per thread and
// row on the way in, whole segments on the way out), thread t computes sub-tensor t of the strip
// from LDS with its block in registers, and the results go back through LDS: as bf16 (ZIN), or as
// float32 from which each thread of the store phase takes one whole segment, finds its largest
// magnitude by itself and writes 32 bytes of halves and the exponent byte (no cross-lane step).
// Two barriers per pair of rows; two pairs are requested ahead; several workgroups share a
// compute unit, so their phases overlap.
// OP: the stage (or chain of stages) on the P coordinates base + j S of a sub-tensor; ZI / ZO:
// block-scaled halves on the way in / out (otherwise bf16).  With halves on both sides (a trip
// between two intermediates) the launch may run in place: a workgroup reads and writes exactly
// the coordinates of its own strip, and requests rows ahead of the ones it writes.
template <class OP, bool ZI, bool ZO>
__global__ __launch_bounds__(256) void harp_stream_z16_lds_kernel(const uint16_t *X, int64_t ldx,
                                                                  uint16_t *Y, int64_t ldy, int64_t n,
                                                                  int rows_per_block,
                                                                  const float *__restrict__ params,
                                                                  int nq, int S, int d) {
  constexpr int P = OP::P, NV = OP::NV;
  constexpr int NP = 32 * P;                  // 16-byte input pieces per row
  constexpr int PPT = (NP + 255) / 256;       // ... per thread (1 or 2)
  static_assert(PPT <= 2 && 4 * P <= 256, "sub-tensors of at most 16 coordinates");
  __shared__ uint16_t s_in[2][P][256];        // the pair's rows as loaded
  __shared__ uint32_t s_ex[2][P][4];          // ZI: their exponent bytes
  __shared__ float s_out[2][P][ZO ? 256 : 128];   // float32 results, or bf16 pairs
  const int t = threadIdx.x;
  const int q0 = blockIdx.x * 256;
  const int hi = q0 / S;
  const unsigned strip = (unsigned)hi * P * S + (unsigned)(q0 - hi * S);   // first coordinate, j = 0
  float prm[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) prm[v] = params[(size_t)v * nq + q0 + t];
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
  const int nr = (int)((r0 + rows_per_block < n) ? rows_per_block : n - r0);
  const int last = nr - 1;
  const uint16_t *xb = X + r0 * ldx;
  uint16_t *yb = Y + r0 * ldy;
  // This thread's input pieces: 8 coordinates of chunk pj at offset pc of the strip, and (ZI)
  // four exponent bytes.  Threads beyond the last piece take the last piece a second time
  // (same address, same value to the same LDS slot), so that no access is conditional.
  // (first piece t, second piece t + 256 where a row has more than 256 pieces; scalars, not
  // arrays: arrays passed to the helpers below by reference ended up in scratch memory)
  const int tpa = t < NP ? t : NP - 1, tpb = (t + 256) < NP ? (t + 256) : NP - 1;
  const int pja = tpa >> 5, pca = (tpa & 31) * 8, pjb = tpb >> 5, pcb = (tpb & 31) * 8;
  const unsigned poffa = strip + (unsigned)pja * S + pca, poffb = strip + (unsigned)pjb * S + pcb;
  const int te = t < 4 * P ? t : 4 * P - 1;
  const unsigned eoff = (strip + (unsigned)(te >> 2) * S) / 16 + 4 * (te & 3);
  // pairs k and k + 1 in named registers
  uint4 a0, a1, b0, b1, a0x, a1x, b0x, b1x;   // ..x: the second piece (PPT == 2)
  a0x = a1x = b0x = b1x = make_uint4(0u, 0u, 0u, 0u);
  uint32_t ea0 = 0, ea1 = 0, eb0 = 0, eb1 = 0;
  auto request = [&](int pair, uint4 &w0, uint4 &w1, uint4 &w0x, uint4 &w1x, uint32_t &e0, uint32_t &e1) {
    const int r = 2 * pair;
    const uint16_t *x0 = xb + (int64_t)(r < last ? r : last) * ldx;   // past the end: the last row again
    const uint16_t *x1 = xb + (int64_t)(r + 1 < last ? r + 1 : last) * ldx;
    w0 = *reinterpret_cast<const uint4 *>(x0 + poffa);
    w1 = *reinterpret_cast<const uint4 *>(x1 + poffa);
    if constexpr (PPT == 2) {
      w0x = *reinterpret_cast<const uint4 *>(x0 + poffb);
      w1x = *reinterpret_cast<const uint4 *>(x1 + poffb);
    }
    if constexpr (ZI) {
      e0 = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint8_t *>(x0 + d) + eoff);
      e1 = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint8_t *>(x1 + d) + eoff);
    }
  };
  auto stage = [&](const uint4 &w0, const uint4 &w1, const uint4 &w0x, const uint4 &w1x, uint32_t e0,
                   uint32_t e1) {
    *reinterpret_cast<uint4 *>(&s_in[0][pja][pca]) = w0;
    *reinterpret_cast<uint4 *>(&s_in[1][pja][pca]) = w1;
    if constexpr (PPT == 2) {
      *reinterpret_cast<uint4 *>(&s_in[0][pjb][pcb]) = w0x;
      *reinterpret_cast<uint4 *>(&s_in[1][pjb][pcb]) = w1x;
    }
    if constexpr (ZI) {
      s_ex[0][te >> 2][te & 3] = e0;
      s_ex[1][te >> 2][te & 3] = e1;
    }
  };
  auto compute = [&]() {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float x[P];
#pragma unroll
      for (int j = 0; j < P; ++j) {
        const uint32_t v = s_in[h][j][t];
        if (ZI) {
          const uint32_t ex = reinterpret_cast<const uint8_t *>(&s_ex[h][j][0])[t >> 4];
          x[j] = (float)__builtin_bit_cast(_Float16, (uint16_t)v) * z16_up(ex);
        } else {
          x[j] = __uint_as_float(v << 16);
        }
      }
      OP::apply(x, prm);
#pragma unroll
      for (int j = 0; j < P; ++j) {
        if (ZO) s_out[h][j][t] = x[j];
        else reinterpret_cast<uint16_t *>(&s_out[h][j][0])[t] = narrow_bf16(x[j]);
      }
    }
  };
  auto put = [&](int pair) {
    if (!ZO) {
      // 16-byte pieces of bf16: 2 rows x P chunks x 32 pieces
      for (int p = t; p < 2 * NP; p += 256) {
        const int h = p / NP, pp = p - h * NP, j = pp >> 5, c = (pp & 31) * 8;
        const int r = 2 * pair + h;
        if (r < nr)
          *reinterpret_cast<uint4 *>(yb + (int64_t)r * ldy + strip + (unsigned)j * S + c) =
              *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(&s_out[h][j][0]) + c);
      }
    } else {
      // whole segments: 2 rows x P chunks x 16 segments of 16 float32 results
      for (int sg = t; sg < 2 * 16 * P; sg += 256) {
        const int h = sg / (16 * P), ss = sg - h * 16 * P, j = ss >> 4, c = (ss & 15) * 16;
        const int r = 2 * pair + h;
        float v[16];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float4 f = *reinterpret_cast<const float4 *>(&s_out[h][j][c + 4 * k]);
          v[4 * k] = f.x; v[4 * k + 1] = f.y; v[4 * k + 2] = f.z; v[4 * k + 3] = f.w;
        }
        float mx = fabsf(v[0]);
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, fabsf(v[e]));
        const uint32_t ex = z16_exponent(mx);
        const float f = z16_down(ex);
        if (r < nr) {
          uint16_t *yr = yb + (int64_t)r * ldy;
          const unsigned co = strip + (unsigned)j * S + c;
#pragma unroll
          for (int k = 0; k < 2; ++k)
            *reinterpret_cast<uint4 *>(yr + co + 8 * k) =
                make_uint4(z16_pack(v[8 * k] * f, v[8 * k + 1] * f), z16_pack(v[8 * k + 2] * f, v[8 * k + 3] * f),
                           z16_pack(v[8 * k + 4] * f, v[8 * k + 5] * f), z16_pack(v[8 * k + 6] * f, v[8 * k + 7] * f));
          reinterpret_cast<uint8_t *>(yr + d)[co >> 4] = (uint8_t)ex;
        }
      }
    }
  };
  const int npairs = (nr + 1) >> 1;
  request(0, a0, a1, a0x, a1x, ea0, ea1);
  request(1, b0, b1, b0x, b1x, eb0, eb1);
  stage(a0, a1, a0x, a1x, ea0, ea1);
  __syncthreads();
  for (int k = 0; k < npairs; k += 2) {
    request(k + 2, a0, a1, a0x, a1x, ea0, ea1);   // pair k is staged already
    compute();                                    // pair k: s_in -> s_out
    __syncthreads();                              // s_out complete, s_in free
    put(k);
    stage(b0, b1, b0x, b1x, eb0, eb1);            // pair k + 1
    __syncthreads();                              // s_in complete, s_out free
    if (k + 1 >= npairs) break;
    request(k + 3, b0, b1, b0x, b1x, eb0, eb1);
    compute();
    __syncthreads();
    put(k + 1);
    stage(a0, a1, a0x, a1x, ea0, ea1);
    __syncthreads();
  }
}

// run-time radix (9..64): parameters are re-read for every row (slow, correctness path)
template <int BMAX>
__global__ __launch_bounds__(256) void harp_stream_generic_kernel(
    const void *__restrict__ X, int64_t ldx, int in_bf16, void *__restrict__ Y, int64_t ldy,
    int out_bf16, int64_t n, int rows_per_block, PassDesc pd) {
  const int nq = pd.nq, S = pd.S, b = pd.b;
  const int q = blockIdx.x * 256 + threadIdx.x;
  if (q >= nq) return;
  const int hi = q / S, lo = q - hi * S;
  const int64_t base = (int64_t)hi * b * S + lo;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
  const int64_t r1 = (r0 + rows_per_block < n) ? r0 + rows_per_block : n;
  for (int64_t row = r0; row < r1; ++row) {
    float x[BMAX];
#pragma unroll
    for (int r = 0; r < BMAX; ++r) {
      const float v = stream_load(X, row * ldx + base + (int64_t)(r < b ? r : b - 1) * S, in_bf16);
      x[r] = (r < b) ? v : 0.0f;
    }
    for (int r2 = 0; r2 < b; ++r2) {
      const float *pp = pd.params + (size_t)r2 * nq + q;
      float acc = 0.0f;
#pragma unroll
      for (int r = 0; r < BMAX; ++r)   // unconditional loads (x[r] is zero past the radix)
        acc = fmaf(x[r], pp[(size_t)(r < b ? r : b - 1) * b * nq], acc);
      stream_store(Y, row * ldy + base + (int64_t)r2 * S, out_bf16, acc);
    }
  }
}

// grid of the streamed kernels: x = blocks of 256 sub-tensors, y = blocks of rows
struct StreamGrid {
  unsigned gx, gy;
  int rpb;
};
StreamGrid stream_grid(int items, const harp_plan *plan, int64_t n) {
  const unsigned gx = (unsigned)((items + 255) / 256);
  // about 8 workgroups per compute unit (occupancy hides the load latency), >= 4 rows each
  const int wgs = 8, minrows = 4;
  int64_t gy = ((int64_t)plan->num_cu * wgs + gx - 1) / gx;
  if (gy > (n + minrows - 1) / minrows) gy = (n + minrows - 1) / minrows;
  if (gy < 1) gy = 1;
  if (gy > 65535) gy = 65535;
  const int rpb = (int)((n + gy - 1) / gy);
  gy = (n + rpb - 1) / rpb;
  return StreamGrid{gx, (unsigned)gy, rpb};
}

template <class KERN>
harp_status_t launch_stream_grid(KERN kern, int items, const harp_plan *plan, const PassDesc &pd,
                                 const void *X, int64_t ldx, int in_bf16, void *Y, int64_t ldy,
                                 int out_bf16, int64_t n, hipStream_t stream) {
  const StreamGrid g = stream_grid(items, plan, n);
  hipLaunchKernelGGL(kern, dim3(g.gx, g.gy), dim3(256), 0, stream, X, ldx, in_bf16, Y, ldy,
                     out_bf16, n, g.rpb, pd);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

template <class OP, typename TI, typename TO>
harp_status_t launch_stream_typed(const harp_plan *plan, const PassDesc &pd, const void *X,
                                  int64_t ldx, void *Y, int64_t ldy, int64_t n,
                                  hipStream_t stream) {
  const StreamGrid g = stream_grid(pd.nq, plan, n);
  hipLaunchKernelGGL((harp_stream_kernel<OP, TI, TO>), dim3(g.gx, g.gy), dim3(256), 0, stream,
                     (const TI *)X, ldx, (TO *)Y, ldy, n, g.rpb, pd.params, pd.nq, pd.S);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

// A streamed pass is never both the first and the last segment of a split program, so bf16 on
// both sides does not occur.
template <class OP>
harp_status_t launch_stream_op(const harp_plan *plan, const PassDesc &pd, const void *X,
                               int64_t ldx, int ib, void *Y, int64_t ldy, int ob, int64_t n,
                               hipStream_t stream) {
  if ((int64_t)pd.P * pd.S >= (int64_t)1 << 31) return HARP_ERR_UNSUPPORTED;
  if (ib && !ob) return launch_stream_typed<OP, uint16_t, float>(plan, pd, X, ldx, Y, ldy, n, stream);
  if (!ib && ob) return launch_stream_typed<OP, float, uint16_t>(plan, pd, X, ldx, Y, ldy, n, stream);
  if (!ib && !ob) return launch_stream_typed<OP, float, float>(plan, pd, X, ldx, Y, ldy, n, stream);
  return HARP_ERR_UNSUPPORTED;
}

// dense stage of radix 3..8 between a bf16 side and the block-scaled half intermediate
template <class OP>
harp_status_t launch_stream_z16_lds(const harp_plan *plan, const PassDesc &pd, const void *X,
                                    int64_t ldx, void *Y, int64_t ldy, int64_t n, bool zin, bool zout,
                                    hipStream_t stream) {
  const unsigned gx = (unsigned)(pd.nq / 256);
  // about 8 workgroups per compute unit, rows in pairs, at least 8 rows each
  int64_t gy = ((int64_t)plan->num_cu * 8 + gx - 1) / gx;
  if (gy > (n + 7) / 8) gy = (n + 7) / 8;
  if (gy < 1) gy = 1;
  if (gy > 65535) gy = 65535;
  int64_t rpb = (n + gy - 1) / gy;
  rpb = (rpb + 1) / 2 * 2;
  gy = (n + rpb - 1) / rpb;
#define HARP_Z16_LDS(ZI_, ZO_)                                                                            \
  hipLaunchKernelGGL((harp_stream_z16_lds_kernel<OP, ZI_, ZO_>), dim3(gx, (unsigned)gy), dim3(256), 0,     \
                     stream, (const uint16_t *)X, ldx, (uint16_t *)Y, ldy, n, (int)rpb, pd.params, pd.nq, \
                     pd.S, (int)plan->d)
  if (zin && zout) HARP_Z16_LDS(true, true);
  else if (zin) HARP_Z16_LDS(true, false);
  else if (zout) HARP_Z16_LDS(false, true);
  else return HARP_ERR_UNSUPPORTED;
#undef HARP_Z16_LDS
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

// whether the LDS-staged kernel can run this pass (strides and strips of whole 256-coordinate
// runs, 16-byte aligned rows)
bool z16_lds_ok(const harp_plan *plan, const PassDesc &pd, const void *X, int64_t ldx, const void *Y,
                int64_t ldy) {
  return pd.S % 256 == 0 && pd.nq % 256 == 0 && ldx % 8 == 0 && ldy % 8 == 0 && (uintptr_t)X % 16 == 0 &&
         (uintptr_t)Y % 16 == 0 && plan->d % 64 == 0;
}

template <class OP>
harp_status_t launch_stream_z16_op(const harp_plan *plan, const PassDesc &pd, const void *X,
                                   int64_t ldx, void *Y, int64_t ldy, int64_t n, bool zin, bool zout,
                                   hipStream_t stream) {
  // Writing the halves (the stage runs first), or halves on both sides: the LDS-staged kernel
  // (2048 x 14336: 37.5 -> 30 us).  Reading them into bf16, the two kernels measured within 3 %
  // of each other (radix 3 and 28672 faster from registers, 14336 from LDS): the register kernel.
  const bool lds_ok = z16_lds_ok(plan, pd, X, ldx, Y, ldy);
  if (zout && lds_ok) return launch_stream_z16_lds<OP>(plan, pd, X, ldx, Y, ldy, n, zin, zout, stream);
  if (zin && zout) return HARP_ERR_UNSUPPORTED;
  const StreamGrid g = stream_grid(pd.nq / 2, plan, n);
  if (zin)
    hipLaunchKernelGGL((harp_stream_z16_kernel<OP, true>), dim3(g.gx, g.gy), dim3(256), 0, stream,
                       (const uint16_t *)X, ldx, (uint16_t *)Y, ldy, n, g.rpb, pd.params, pd.nq, pd.S,
                       (int)plan->d);
  else
    hipLaunchKernelGGL((harp_stream_z16_kernel<OP, false>), dim3(g.gx, g.gy), dim3(256), 0, stream,
                       (const uint16_t *)X, ldx, (uint16_t *)Y, ldy, n, g.rpb, pd.params, pd.nq, pd.S,
                       (int)plan->d);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

template <bool DESC, int FORM>
harp_status_t launch_stream_pow2(const harp_plan *plan, const PassDesc &pd, const void *X,
                                 int64_t ldx, int ib, void *Y, int64_t ldy, int ob, int64_t n,
                                 hipStream_t st) {
  switch (pd.k) {
    case 1: return launch_stream_op<OpPow2<1, DESC, FORM>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, st);
    case 2: return launch_stream_op<OpPow2<2, DESC, FORM>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, st);
    case 3: return launch_stream_op<OpPow2<3, DESC, FORM>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, st);
    case 4:
      if (FORM != 0)
        return launch_stream_op<OpPow2<4, DESC, (FORM == 0 ? 1 : FORM)>>(plan, pd, X, ldx, ib, Y,
                                                                        ldy, ob, n, st);
      return HARP_ERR_UNSUPPORTED;
    default: return HARP_ERR_UNSUPPORTED;
  }
}

// ------------------------------------------------------------------------------------------
// dst[c, r] = src[r, c] with conversion; 32 x 32 tiles through LDS.
template <typename TS, typename TD>
__global__ __launch_bounds__(256) void harp_transpose_kernel(const TS *__restrict__ src, int64_t lds_,
                                                             TD *__restrict__ dst, int64_t ldd,
                                                             int64_t rows, int64_t cols) {
  __shared__ float buf[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  const int64_t c0 = (int64_t)blockIdx.x * 32, r0 = (int64_t)blockIdx.y * 32;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int64_t r = r0 + ty + 8 * k, c = c0 + tx;
    if (r < rows && c < cols) buf[ty + 8 * k][tx] = load_one(src + r * lds_ + c);
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int64_t c = c0 + ty + 8 * k, r = r0 + tx;
    if (r < rows && c < cols) store_one(dst + c * ldd + r, buf[tx][ty + 8 * k]);
  }
}

// Four consecutive elements at p (16-byte aligned for float, 8-byte for bf16).
__device__ __forceinline__ void load_four(const float *p, float (&v)[4]) {
  const float4 f = *reinterpret_cast<const float4 *>(p);
  v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
}
__device__ __forceinline__ void load_four(const uint16_t *p, float (&v)[4]) {
  const uint2 w = *reinterpret_cast<const uint2 *>(p);
  v[0] = __uint_as_float(w.x << 16); v[1] = __uint_as_float(w.x & 0xffff0000u);
  v[2] = __uint_as_float(w.y << 16); v[3] = __uint_as_float(w.y & 0xffff0000u);
}
__device__ __forceinline__ void store_four(float *p, const float (&v)[4]) {
  *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store_four(uint16_t *p, const float (&v)[4]) {
  *reinterpret_cast<uint2 *>(p) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}

// The same on 64 x 64 tiles with four elements per access on both sides (256-byte runs of a
// float row); leading dimensions multiples of 4 and 16-byte aligned bases.  Vectors that
// cross the matrix edge fall back to single elements.
template <typename TS, typename TD>
__global__ __launch_bounds__(256) void harp_transpose64_kernel(const TS *__restrict__ src,
                                                               int64_t lds_, TD *__restrict__ dst,
                                                               int64_t ldd, int64_t rows,
                                                               int64_t cols) {
  __shared__ float buf[64][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;   // 16 vectors x 16 rows per sweep
  const int64_t c0 = (int64_t)blockIdx.x * 64, r0 = (int64_t)blockIdx.y * 64;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int lr = ty + 16 * k;
    const int64_t r = r0 + lr, c = c0 + 4 * tx;
    if (r < rows) {
      if (c + 3 < cols) {
        float v[4];
        load_four(src + r * lds_ + c, v);
#pragma unroll
        for (int i = 0; i < 4; ++i) buf[lr][4 * tx + i] = v[i];
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (c + i < cols) buf[lr][4 * tx + i] = load_one(src + r * lds_ + c + i);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int lc = ty + 16 * k;
    const int64_t c = c0 + lc, r = r0 + 4 * tx;
    if (c < cols) {
      if (r + 3 < rows) {
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = buf[4 * tx + i][lc];
        store_four(dst + c * ldd + r, v);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (r + i < rows) store_one(dst + c * ldd + r + i, buf[4 * tx + i][lc]);
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void harp_copy2d_kernel(const T *__restrict__ src, int64_t lds_,
                                                          T *__restrict__ dst, int64_t ldd,
                                                          int64_t rows, int64_t cols) {
  const int64_t total = rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / cols, c = i - r * cols;
    dst[r * ldd + c] = src[r * lds_ + c];
  }
}

// Plain copy of a row-major matrix whose rows are whole 16-byte pieces at 16-byte aligned
// addresses: four pieces per thread, all four loads issued before the first store.  rowp =
// pieces per row, lds16 / ldd16 = leading dimensions in pieces.
__global__ __launch_bounds__(256) void harp_copy2d_vec_kernel(const uint4 *__restrict__ src,
                                                              uint32_t lds16, uint4 *__restrict__ dst,
                                                              uint32_t ldd16, uint32_t rowp,
                                                              uint32_t total) {
  const uint32_t i0 = blockIdx.x * 1024u + threadIdx.x;
  uint4 v[4];
  uint32_t so[4], dof[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    uint32_t i = i0 + 256u * k;
    if (i >= total) i = total - 1;            // clamped: the extra lanes repeat the last piece
    const uint32_t r = i / rowp, c = i - r * rowp;
    so[k] = r * lds16 + c;
    dof[k] = r * ldd16 + c;
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) v[k] = src[so[k]];
#pragma unroll
  for (int k = 0; k < 4; ++k) dst[dof[k]] = v[k];
}

template <typename TI, typename TO>
harp_status_t launch_tile_typed(const harp_plan *plan, const Program *dprog, int p0, int p1,
                                int chunk, const void *X, int64_t ldx, void *Y, int64_t ldy,
                                int64_t n, hipStream_t stream) {
  const int d = chunk;
  const int nchunk = (int)(plan->d / chunk);
  const LaunchCfg cfg = choose_launch(plan, chunk, n * nchunk);
  if (cfg.rows_per_tile < 1) return HARP_ERR_UNSUPPORTED;
  const size_t lds = (size_t)cfg.rows_per_tile * d * sizeof(float);
  auto kern = harp_tile_kernel<TI, TO>;
  static thread_local int attr_done_dev = -1;
  if (attr_done_dev != plan->device) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            plan->lds_bytes) != hipSuccess)
      (void)hipGetLastError();  // not fatal below 64 KB; a too-large launch fails cleanly later
    attr_done_dev = plan->device;
  }
  constexpr int VI = IoTraits<TI>::kVec, VO = IoTraits<TO>::kVec;
  const int vec_in = (d % VI == 0) && (ldx % VI == 0) && ((uintptr_t)X % 16 == 0);
  const int vec_out = (d % VO == 0) && (ldy % VO == 0) && ((uintptr_t)Y % 16 == 0);
  const int64_t tiles = ((n + cfg.rows_per_tile - 1) / cfg.rows_per_tile) * nchunk;
  if (tiles > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(cfg.threads), lds, stream,
                     (const TI *)X, ldx, (TO *)Y, ldy, n, d, nchunk, cfg.rows_per_tile, vec_in,
                     vec_out, dprog, p0, p1);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

template <typename TS, typename TD>
harp_status_t launch_transpose_typed(const void *src, int64_t lds_, void *dst, int64_t ldd,
                                     int64_t rows, int64_t cols, hipStream_t stream) {
  if ((rows + 31) / 32 > 65535 * 16) return HARP_ERR_UNSUPPORTED;
  if (lds_ % 4 == 0 && ldd % 4 == 0 && (uintptr_t)src % 16 == 0 && (uintptr_t)dst % 16 == 0) {
    const dim3 grid64((unsigned)((cols + 63) / 64), (unsigned)((rows + 63) / 64));
    hipLaunchKernelGGL((harp_transpose64_kernel<TS, TD>), grid64, dim3(256), 0, stream,
                       (const TS *)src, lds_, (TD *)dst, ldd, rows, cols);
    return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
  }
  const dim3 grid((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32));
  hipLaunchKernelGGL((harp_transpose_kernel<TS, TD>), grid, dim3(256), 0, stream, (const TS *)src,
                     lds_, (TD *)dst, ldd, rows, cols);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}


}  // namespace

// d = coordinates per on-chip row (chunk), n = number of such rows in the launch
LaunchCfg choose_launch(const harp_plan *plan, int64_t d, int64_t n) {
  LaunchCfg cfg{0, 256};
  const int rmax = (int)(plan->lds_bytes / (4 * d));   // rows of the tile that fit in LDS
  if (rmax < 1) return cfg;
  // 8 rows per tile, more for short chunks so that the parameters a tile reads (they are as
  // many as one row has coordinates, per stage) are reused by at least 16K coordinates
  int rwant = (int)(16384 / d);
  if (rwant < 8) rwant = 8;
  if (rwant > 64) rwant = 64;
  int R = plan->rows_override > 0 ? plan->rows_override : (rmax < rwant ? rmax : rwant);
  if (R > rmax) R = rmax;
  if (plan->rows_override == 0) {
    // keep every compute unit busy: shrink the tile while there are fewer tiles than CUs
    while (R > 1 && (n + R - 1) / R < plan->num_cu) R = (R + 1) / 2;
  }
  cfg.rows_per_tile = R;
  const int64_t work = (int64_t)R * d / 16;
  int nt = 256;
  while (nt < 512 && nt < work) nt *= 2;
  if (nt < 64) nt = 64;
  if (nt > 512) nt = 512;
  nt = (nt / 64) * 64;
  cfg.threads = nt;
  return cfg;
}

harp_status_t launch_tile_kernel(const harp_plan *plan, const Program *prog, int p0, int p1,
                                 int chunk, const void *X, int64_t ldx, harp_dtype_t dt_in,
                                 void *Y, int64_t ldy, harp_dtype_t dt_out, int64_t n,
                                 hipStream_t stream) {
  if (n == 0) return HARP_OK;
  if (chunk < 1 || plan->d % chunk != 0 || (int64_t)chunk * 4 > plan->lds_bytes)
    return HARP_ERR_UNSUPPORTED;
  if (dt_in == HARP_F32 && dt_out == HARP_F32)
    return launch_tile_typed<float, float>(plan, prog, p0, p1, chunk, X, ldx, Y, ldy, n, stream);
  if (dt_in == HARP_BF16 && dt_out == HARP_BF16)
    return launch_tile_typed<uint16_t, uint16_t>(plan, prog, p0, p1, chunk, X, ldx, Y, ldy, n,
                                                 stream);
  if (dt_in == HARP_BF16 && dt_out == HARP_F32)
    return launch_tile_typed<uint16_t, float>(plan, prog, p0, p1, chunk, X, ldx, Y, ldy, n,
                                              stream);
  return launch_tile_typed<float, uint16_t>(plan, prog, p0, p1, chunk, X, ldx, Y, ldy, n, stream);
}

// the streamed stage has a kernel for the block-scaled half intermediate: one dense stage of
// radix 3..8 whose stride is a multiple of 16, rows that allow 32-bit accesses
bool stream_z16_supported(const PassDesc &pd, const void *X, int64_t ldx, const void *Y,
                          int64_t ldy) {
  const bool chain = (pd.kind == PASS_SMALL_CHAIN && pd.b == 3 && pd.k == 2);   // LDS-staged kernel only
  // one dense radix-2 stage: its four values per block lie in the image like a radix-2 "small" stage
  const bool dense2 = (pd.kind == PASS_POW2_DENSE && pd.k == 1 && pd.P == 2 && pd.V == 4);
  if (!chain && !dense2 && (pd.kind != PASS_SMALL || pd.b < 3 || pd.b > 8)) return false;
  if (pd.tied) return false;
  if (chain && (pd.S % 256 != 0 || pd.nq % 256 != 0 || ldx % 8 || ldy % 8 || (uintptr_t)X % 16 ||
                (uintptr_t)Y % 16))
    return false;
  if (pd.S % 16 != 0 || (pd.nq & 1)) return false;
  if ((ldx % 2) || (ldy % 2) || ((uintptr_t)X % 4) || ((uintptr_t)Y % 4)) return false;
  if ((int64_t)pd.P * pd.S >= (int64_t)1 << 31) return false;
  return true;
}

harp_status_t launch_stream_pass(const harp_plan *plan, const HostProgram &hp, int p,
                                 const void *X, int64_t ldx, harp_dtype_t dt_in, void *Y,
                                 int64_t ldy, harp_dtype_t dt_out, int64_t n, bool allow_narrow,
                                 hipStream_t stream) {
  if (n == 0) return HARP_OK;
  const PassDesc &pd = hp.prog.pass[p];
  if (!plan->no_mfma && mfma_pass_supported(pd, X, ldx, Y, ldy))
    return launch_mfma_pass(plan, pd, X, ldx, dt_in, Y, ldy, dt_out, n, allow_narrow, stream);
  if (pd.tied) return HARP_ERR_UNSUPPORTED;   // only the matrix-core kernel reads a tied table
  if ((int)dt_in == kDtZ16 || (int)dt_out == kDtZ16) {
    if (!stream_z16_supported(pd, X, ldx, Y, ldy)) return HARP_ERR_UNSUPPORTED;
    const bool zin = (int)dt_in == kDtZ16, zout = (int)dt_out == kDtZ16;
    if ((!zin && dt_in != HARP_BF16) || (!zout && dt_out != HARP_BF16)) return HARP_ERR_UNSUPPORTED;
    if (zin && zout && !z16_lds_ok(plan, pd, X, ldx, Y, ldy)) return HARP_ERR_UNSUPPORTED;
    if (pd.kind == PASS_SMALL_CHAIN) {
      if (!z16_lds_ok(plan, pd, X, ldx, Y, ldy)) return HARP_ERR_UNSUPPORTED;
      return pd.desc ? launch_stream_z16_lds<OpSmallChain<3, 2, true>>(plan, pd, X, ldx, Y, ldy, n, zin, zout, stream)
                     : launch_stream_z16_lds<OpSmallChain<3, 2, false>>(plan, pd, X, ldx, Y, ldy, n, zin, zout, stream);
    }
    switch (pd.b) {
      case 2: return launch_stream_z16_op<OpSmall<2>>(plan, pd, X, ldx, Y, ldy, n, zin, zout, stream);
      case 3: return launch_stream_z16_op<OpSmall<3>>(plan, pd, X, ldx, Y, ldy, n, zin, zout, stream);
      case 4: return launch_stream_z16_op<OpSmall<4>>(plan, pd, X, ldx, Y, ldy, n, zin, zout, stream);
      case 5: return launch_stream_z16_op<OpSmall<5>>(plan, pd, X, ldx, Y, ldy, n, zin, zout, stream);
      case 6: return launch_stream_z16_op<OpSmall<6>>(plan, pd, X, ldx, Y, ldy, n, zin, zout, stream);
      case 7: return launch_stream_z16_op<OpSmall<7>>(plan, pd, X, ldx, Y, ldy, n, zin, zout, stream);
      default: return launch_stream_z16_op<OpSmall<8>>(plan, pd, X, ldx, Y, ldy, n, zin, zout, stream);
    }
  }
  const int ib = dt_in == HARP_BF16, ob = dt_out == HARP_BF16;
  switch (pd.kind) {
    case PASS_POW2_DENSE:
      return pd.desc ? launch_stream_pow2<true, 0>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream)
                     : launch_stream_pow2<false, 0>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
    case PASS_POW2_LIFT:
      return pd.desc ? launch_stream_pow2<true, 1>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream)
                     : launch_stream_pow2<false, 1>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
    case PASS_POW2_LIFT_LD:
      return pd.desc ? launch_stream_pow2<true, 2>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream)
                     : launch_stream_pow2<false, 2>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
    case PASS_POW2_SCALED:
      return pd.desc ? launch_stream_pow2<true, 3>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream)
                     : launch_stream_pow2<false, 3>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
    case PASS_POW2_SCALED_LD:
      return pd.desc ? launch_stream_pow2<true, 4>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream)
                     : launch_stream_pow2<false, 4>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
    case PASS_SMALL_CHAIN:
      if (pd.b != 3) return HARP_ERR_UNSUPPORTED;
      if (pd.k == 2)
        return pd.desc ? launch_stream_op<OpSmallChain<3, 2, true>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream)
                       : launch_stream_op<OpSmallChain<3, 2, false>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
      // three stages per trip (27 coordinates and 243 block values per thread) were measured
      // too: the kernel needs the whole register file and is slower than two trips
      return HARP_ERR_UNSUPPORTED;
    case PASS_SMALL:
      switch (pd.b) {
        case 3: return launch_stream_op<OpSmall<3>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
        case 4: return launch_stream_op<OpSmall<4>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
        case 5: return launch_stream_op<OpSmall<5>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
        case 6: return launch_stream_op<OpSmall<6>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
        case 7: return launch_stream_op<OpSmall<7>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
        case 8: return launch_stream_op<OpSmall<8>>(plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
        default: return HARP_ERR_UNSUPPORTED;
      }
    default:
      if (pd.b <= 16)
        return launch_stream_grid(harp_stream_generic_kernel<16>, pd.nq, plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
      return launch_stream_grid(harp_stream_generic_kernel<64>, pd.nq, plan, pd, X, ldx, ib, Y, ldy, ob, n, stream);
  }
}

harp_status_t launch_transpose(const void *src, int64_t lds_, harp_dtype_t dt_src, void *dst,
                               int64_t ldd, harp_dtype_t dt_dst, int64_t rows, int64_t cols,
                               hipStream_t stream) {
  if (rows == 0 || cols == 0) return HARP_OK;
  if (dt_src == HARP_F32 && dt_dst == HARP_F32)
    return launch_transpose_typed<float, float>(src, lds_, dst, ldd, rows, cols, stream);
  if (dt_src == HARP_BF16 && dt_dst == HARP_F32)
    return launch_transpose_typed<uint16_t, float>(src, lds_, dst, ldd, rows, cols, stream);
  if (dt_src == HARP_F32 && dt_dst == HARP_BF16)
    return launch_transpose_typed<float, uint16_t>(src, lds_, dst, ldd, rows, cols, stream);
  return launch_transpose_typed<uint16_t, uint16_t>(src, lds_, dst, ldd, rows, cols, stream);
}

harp_status_t launch_copy2d(const void *src, int64_t lds_, void *dst, int64_t ldd, int64_t rows,
                            int64_t cols, harp_dtype_t dt, hipStream_t stream) {
  if (rows == 0 || cols == 0) return HARP_OK;
  const int64_t total = rows * cols;
  const int64_t es = dt == HARP_F32 ? 4 : 2;
  // rows of whole, aligned 16-byte pieces and 32-bit piece offsets: the vector kernel
  if ((cols * es) % 16 == 0 && (lds_ * es) % 16 == 0 && (ldd * es) % 16 == 0 &&
      (uintptr_t)src % 16 == 0 && (uintptr_t)dst % 16 == 0 && src != dst &&
      rows * std::max(lds_, ldd) * es / 16 < ((int64_t)1 << 32)) {
    const int64_t rowp = cols * es / 16, pieces = rows * rowp;
    hipLaunchKernelGGL(harp_copy2d_vec_kernel, dim3((unsigned)((pieces + 1023) / 1024)), dim3(256), 0,
                       stream, (const uint4 *)src, (uint32_t)(lds_ * es / 16), (uint4 *)dst,
                       (uint32_t)(ldd * es / 16), (uint32_t)rowp, (uint32_t)pieces);
    return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
  }
  int64_t blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (dt == HARP_F32)
    hipLaunchKernelGGL((harp_copy2d_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, stream,
                       (const float *)src, lds_, (float *)dst, ldd, rows, cols);
  else
    hipLaunchKernelGGL((harp_copy2d_kernel<uint16_t>), dim3((unsigned)blocks), dim3(256), 0,
                       stream, (const uint16_t *)src, lds_, (uint16_t *)dst, ldd, rows, cols);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

}  // namespace harp
