// Backward of Y = X U with respect to the block kernels and to X -- the gradient that the
// update of the layerwise fitting procedure (Algorithm 3) needs, by the chain rule through
// Algorithm 1.  With x_0 = X diag(sigma), x_{t+1} = stage_t(x_t) and g_m = G = dL/dY:
//     dK_t[c] = sum over rows of x_t[idx]^T g_{t+1}[idx],     g_t[idx] = g_{t+1}[idx] K_t[c]^T,
// idx = the b_t coordinates alpha b s + r s + beta of block c = alpha s + beta, and dX = g_0
// diag(sigma).  Nothing is assumed about the blocks (they need not be orthogonal).
//
// First version, stage by stage through device memory: the forward pass keeps the input of
// every stage (m float32 copies of the batch in the workspace), the backward pass runs one kernel
// per stage that updates g in place and leaves per-row-chunk partial sums of dK, and a
// reduction kernel adds the chunks in a fixed order (no atomics: results are reproducible).
// One thread owns one block c for a chunk of rows: its b*b kernel values and b*b accumulators
// stay in registers.  Up to three consecutive radix-2 stages share one kernel: a thread owns
// the 2^k coordinates base + e s and the k 2^(k-1) blocks that act on them, the forward kernel
// stores only the run's output, and the backward kernel recomputes the run's inner activations
// in registers.  Radices up to 8 (the plan's dense per-stage image with the signs folded into
// stage 0 is the one the column-mode passes use).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <vector>

#include "harp_internal.h"

namespace harp {
namespace {

constexpr int kGradThreads = 256;

__device__ __forceinline__ float grad_widen(float v) { return v; }
__device__ __forceinline__ float grad_widen(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ void grad_narrow(float v, float *p) { *p = v; }
__device__ __forceinline__ void grad_narrow(float v, uint16_t *p) {
  const uint32_t u = __float_as_uint(v);
  const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  const uint32_t quiet = (u >> 16) | 0x40u;
  *p = (uint16_t)(((u & 0x7fffffffu) > 0x7f800000u) ? quiet : rounded);
}

// dst[r, c] = convert(src[r, c]); VEC: eight elements per thread with 16-byte accesses on the
// two-byte side (d a multiple of 8, rows and pointers on 16-byte boundaries)
template <typename TS, typename TD, bool VEC>
__global__ __launch_bounds__(kGradThreads) void harp_grad_convert_kernel(
    const TS *__restrict__ src, int64_t lds_, TD *__restrict__ dst, int64_t ldd, int64_t n, int d) {
  const int64_t row = blockIdx.y;
  if (VEC) {
    for (int c = 8 * (blockIdx.x * kGradThreads + threadIdx.x); c < d; c += 8 * gridDim.x * kGradThreads) {
      float v[8];
      const TS *sp = src + row * lds_ + c;
      TD *dp = dst + row * ldd + c;
      if (sizeof(TS) == 2) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(sp);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v[2 * i] = __uint_as_float(w[i] << 16);
          v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
      } else {
        const float4 a = *reinterpret_cast<const float4 *>(sp), b = *reinterpret_cast<const float4 *>(sp + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
      }
      if (sizeof(TD) == 2) {
        uint16_t h[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) grad_narrow(v[i], reinterpret_cast<uint16_t *>(&h[i]));
        *reinterpret_cast<uint4 *>(dp) =
            make_uint4(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16),
                       h[4] | ((uint32_t)h[5] << 16), h[6] | ((uint32_t)h[7] << 16));
      } else {
        *reinterpret_cast<float4 *>(dp) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(dp) + 4) = make_float4(v[4], v[5], v[6], v[7]);
      }
    }
  } else {
    for (int c = blockIdx.x * kGradThreads + threadIdx.x; c < d; c += gridDim.x * kGradThreads)
      grad_narrow(grad_widen(src[row * lds_ + c]), dst + row * ldd + c);
  }
  (void)n;
}

// y[idx] = x[idx] K[c] for every row of the chunk blockIdx.y
template <int B>
__global__ __launch_bounds__(kGradThreads) void harp_grad_fwd_kernel(
    const float *__restrict__ X, float *__restrict__ Y, int64_t ld, int64_t n, int rows,
    const float *__restrict__ blocks, int D, int s) {
  const int c = blockIdx.x * kGradThreads + threadIdx.x;
  if (c >= D) return;
  float K[B * B];
#pragma unroll
  for (int v = 0; v < B * B; ++v) K[v] = blocks[(size_t)c * (B * B) + v];
  const int base = (c / s) * B * s + c % s;
  const int64_t r0 = (int64_t)blockIdx.y * rows;
  const int64_t r1 = (r0 + rows < n) ? r0 + rows : n;
  for (int64_t row = r0; row < r1; ++row) {
    const float *x = X + row * ld + base;
    float *y = Y + row * ld + base;
    float v[B];
#pragma unroll
    for (int r = 0; r < B; ++r) v[r] = x[(size_t)r * s];
#pragma unroll
    for (int r2 = 0; r2 < B; ++r2) {
      float acc = 0.f;
#pragma unroll
      for (int r = 0; r < B; ++r) acc = fmaf(v[r], K[r * B + r2], acc);
      y[(size_t)r2 * s] = acc;
    }
  }
}

// For the rows of chunk blockIdx.y: acc[r][r2] += x[idx_r] g[idx_r2];  g[idx_r] <- sum_r2
// g[idx_r2] K[r][r2] (in place).  Partial sums go to partial[(chunk * B*B + v) * D + c].
template <int B>
__global__ __launch_bounds__(kGradThreads) void harp_grad_bwd_kernel(
    const float *__restrict__ X, float *__restrict__ Gm, int64_t ld, int64_t n, int rows,
    const float *__restrict__ blocks, int D, int s, float *__restrict__ partial) {
  const int c = blockIdx.x * kGradThreads + threadIdx.x;
  if (c >= D) return;
  float K[B * B], acc[B * B];
#pragma unroll
  for (int v = 0; v < B * B; ++v) {
    K[v] = blocks[(size_t)c * (B * B) + v];
    acc[v] = 0.f;
  }
  const int base = (c / s) * B * s + c % s;
  const int64_t r0 = (int64_t)blockIdx.y * rows;
  const int64_t r1 = (r0 + rows < n) ? r0 + rows : n;
  for (int64_t row = r0; row < r1; ++row) {
    const float *x = X + row * ld + base;
    float *g = Gm + row * ld + base;
    float xv[B], gv[B];
#pragma unroll
    for (int r = 0; r < B; ++r) {
      xv[r] = x[(size_t)r * s];
      gv[r] = g[(size_t)r * s];
    }
#pragma unroll
    for (int r = 0; r < B; ++r) {
      float back = 0.f;
#pragma unroll
      for (int r2 = 0; r2 < B; ++r2) {
        acc[r * B + r2] = fmaf(xv[r], gv[r2], acc[r * B + r2]);
        back = fmaf(gv[r2], K[r * B + r2], back);
      }
      g[(size_t)r * s] = back;
    }
  }
#pragma unroll
  for (int v = 0; v < B * B; ++v)
    partial[((size_t)blockIdx.y * (B * B) + v) * D + c] = acc[v];
}

// Radix 9..64 (the leftover prime of a schedule): a block no longer fits one thread's registers,
// so thread (c, j) owns one column or row of it.  TR false: y[j] = sum_r x[r] K[r][j] (the stage
// itself); TR true: y[j] = sum_r x[r] K[j][r] (the gradient passed back through it).  Out of
// place.  Workgroup = 64 consecutive blocks c x 4 values of j; blockIdx.z covers the other j.
// BMAX = the radix rounded up to a multiple of 16: the loads of a row are unconditional (index
// clamped to the last coordinate of the block, value replaced by zero), so that all of them are
// in flight together; under a per-load condition each one was waited for before the next was
// issued and the three launches of the radix-43 stage of 11008 took 1 ms each.
template <int BMAX, bool TR>
__global__ __launch_bounds__(kGradThreads) void harp_grad_apply_big_kernel(
    const float *__restrict__ X, float *__restrict__ Y, int64_t ld, int64_t n, int rows,
    const float *__restrict__ blocks, int D, int s, int b) {
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int j = blockIdx.z * 4 + (threadIdx.x >> 6);
  if (c >= D || j >= b) return;
  float kv[BMAX];
  const float *kb = blocks + (size_t)c * b * b;
#pragma unroll
  for (int r = 0; r < BMAX; ++r) {
    const int rc = r < b ? r : b - 1;
    const float v = TR ? kb[j * b + rc] : kb[rc * b + j];
    kv[r] = r < b ? v : 0.f;
  }
  const int base = (c / s) * b * s + c % s;
  const int64_t r0 = (int64_t)blockIdx.y * rows;
  const int64_t r1 = (r0 + rows < n) ? r0 + rows : n;
  for (int64_t row = r0; row < r1; ++row) {
    const float *x = X + row * ld + base;
    float xv[BMAX];
#pragma unroll
    for (int r = 0; r < BMAX; ++r) xv[r] = x[(size_t)(r < b ? r : b - 1) * s];
    float acc = 0.f;
#pragma unroll
    for (int r = 0; r < BMAX; ++r) acc = fmaf(r < b ? xv[r] : 0.f, kv[r], acc);
    Y[row * ld + base + (size_t)j * s] = acc;
  }
}

// Thread (c, r2) accumulates column r2 of dK[c] over the rows of chunk blockIdx.y:
// acc[r] += x[idx_r] g[idx_r2]; partial sums in the layout of the small-radix kernel.
template <int BMAX>
__global__ __launch_bounds__(kGradThreads) void harp_grad_dk_big_kernel(
    const float *__restrict__ X, const float *__restrict__ Gm, int64_t ld, int64_t n, int rows,
    int D, int s, int b, float *__restrict__ partial) {
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int r2 = blockIdx.z * 4 + (threadIdx.x >> 6);
  if (c >= D || r2 >= b) return;
  float acc[BMAX];
#pragma unroll
  for (int r = 0; r < BMAX; ++r) acc[r] = 0.f;
  const int base = (c / s) * b * s + c % s;
  const int64_t r0 = (int64_t)blockIdx.y * rows;
  const int64_t r1 = (r0 + rows < n) ? r0 + rows : n;
  for (int64_t row = r0; row < r1; ++row) {
    const float *x = X + row * ld + base;
    const float gv = Gm[row * ld + base + (size_t)r2 * s];
    float xv[BMAX];
#pragma unroll
    for (int r = 0; r < BMAX; ++r) xv[r] = x[(size_t)(r < b ? r : b - 1) * s];
#pragma unroll
    for (int r = 0; r < BMAX; ++r) acc[r] = fmaf(xv[r], gv, acc[r]);   // r >= b: never stored
  }
#pragma unroll
  for (int r = 0; r < BMAX; ++r)
    if (r < b) partial[((size_t)blockIdx.y * (b * b) + r * b + r2) * D + c] = acc[r];
}

// The same sums on the matrix cores: dK[c] = sum over rows of x[idx]^T g[idx] is a b x rows x b
// product per block (v_mfma_f32_16x16x4_f32, unsplit float32 operands: the k index is the row).
// Needs 16 consecutive blocks to be 16 consecutive coordinates (s a multiple of 16).  A workgroup
// of 16 waves owns 16 consecutive blocks and one row chunk and walks down its rows 8 at a time:
// coalesced 16-byte loads of x and g (next step prefetched in registers) -> two LDS tiles
// [r][block][row] -> wave w multiplies the tiles of its block, KT x KT accumulator tiles in
// registers for the whole chunk.  At the end the accumulators pass through LDS tile by tile
// so that the partial sums leave in runs of 16 consecutive blocks (64 bytes).  Rows past the end
// of the chunk enter as zeros.  Workgroups that share 128-byte lines (two neighbouring block
// tiles) are numbered onto one XCD.
constexpr int kDkRows = 8;                  // rows per step (16 measured 1 % faster at 2048 x 11008 for twice the LDS)
constexpr int kDkLS = kDkRows + 1;          // LDS stride between consecutive blocks
constexpr int kDkJS = 16 * kDkLS + 4;       // LDS stride between consecutive r

template <int KT>
__global__ __launch_bounds__(1024) void harp_grad_dk_mfma_kernel(
    const float *__restrict__ X, const float *__restrict__ Gm, int64_t ld, int64_t n, int rows,
    int D, int s, int b, int gx, int paired, float *__restrict__ partial) {
  typedef float f4v __attribute__((ext_vector_type(4)));
  constexpr int MAXG = (kDkRows * 16 * KT * 4 + 1023) / 1024;
  constexpr int TILE = 16 * KT * kDkJS;
  __shared__ float lds[2 * TILE];
  float *tx = lds, *tg = lds + TILE;
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l = tid & 63, g = l >> 4, c16 = l & 15;
  unsigned wg = blockIdx.x;
  if (paired) {
    const unsigned xcd = wg & 7u, k = wg >> 3;
    wg = ((k >> 1) * 8u + xcd) * 2u + (k & 1u);
  }
  const int qx = (int)(wg % (unsigned)gx), chunk = (int)(wg / (unsigned)gx);
  const int q0 = qx * 16;
  const int64_t base = (int64_t)(q0 / s) * b * s + q0 % s;
  const int64_t r_begin = (int64_t)chunk * rows;
  const int64_t r_end = (r_begin + rows < n) ? r_begin + rows : n;

  const int ngroups = kDkRows * b * 4;   // (row, r, quarter of the 16 blocks) per step
  unsigned off[MAXG];
  int grow[MAXG], slot[MAXG];
#pragma unroll
  for (int u = 0; u < MAXG; ++u) {
    const int gi = (tid + u * 1024) % ngroups;
    const int lo4 = gi & 3, rem = gi >> 2;
    const int row = rem & (kDkRows - 1), j = rem / kDkRows;
    grow[u] = row;
    off[u] = (unsigned)(row * (int)ld + j * s + lo4 * 4);
    slot[u] = j * kDkJS + (lo4 * 4) * kDkLS + row;
  }
  float4 px[MAXG], pg[MAXG];
  auto fetch = [&](int64_t r0, int left) {
    const float *xc = X + r0 * ld + base, *gc = Gm + r0 * ld + base;
    if (left >= kDkRows) {
#pragma unroll
      for (int u = 0; u < MAXG; ++u) {
        px[u] = *reinterpret_cast<const float4 *>(xc + off[u]);
        pg[u] = *reinterpret_cast<const float4 *>(gc + off[u]);
      }
    } else {
#pragma unroll
      for (int u = 0; u < MAXG; ++u) {
        px[u] = pg[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (grow[u] < left) {
          px[u] = *reinterpret_cast<const float4 *>(xc + off[u]);
          pg[u] = *reinterpret_cast<const float4 *>(gc + off[u]);
        }
      }
    }
  };
  auto commit = [&]() {
#pragma unroll
    for (int u = 0; u < MAXG; ++u) {
      float *a = tx + slot[u], *c = tg + slot[u];
      a[0] = px[u].x; a[kDkLS] = px[u].y; a[2 * kDkLS] = px[u].z; a[3 * kDkLS] = px[u].w;
      c[0] = pg[u].x; c[kDkLS] = pg[u].y; c[2 * kDkLS] = pg[u].z; c[3 * kDkLS] = pg[u].w;
    }
  };
  f4v acc[KT][KT];
#pragma unroll
  for (int mt = 0; mt < KT; ++mt)
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) acc[mt][nt] = (f4v){0.f, 0.f, 0.f, 0.f};

  if (r_begin < r_end) {
    fetch(r_begin, (int)(r_end - r_begin));
    for (int64_t r0 = r_begin; r0 < r_end; r0 += kDkRows) {
      commit();
      __syncthreads();
      const int64_t rn = r0 + kDkRows;
      if (rn < r_end) fetch(rn, (int)(r_end - rn));
#pragma unroll
      for (int ks = 0; ks < kDkRows / 4; ++ks) {
        float a[KT], bv[KT];
#pragma unroll
        for (int t = 0; t < KT; ++t) {
          const int j = 16 * t + c16;
          const int at = (j < b ? j : 0) * kDkJS + w * kDkLS + 4 * ks + g;
          a[t] = (j < b) ? tx[at] : 0.f;
          bv[t] = (j < b) ? tg[at] : 0.f;
        }
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
          for (int nt = 0; nt < KT; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[mt], bv[nt], acc[mt][nt], 0, 0, 0);
      }
      __syncthreads();   // every wave has read its operands: the tiles are free again
    }
  }
  // accumulator tile (mt, nt) of all 16 blocks -> LDS [m][n][block] -> 64-byte runs
  float *so = lds;
  const int e = tid >> 2, quarter = tid & 3;
  const int em = e >> 4, en = e & 15;
#pragma unroll
  for (int mt = 0; mt < KT; ++mt)
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
#pragma unroll
      for (int i = 0; i < 4; ++i) so[((4 * g + i) * 16 + c16) * 16 + w] = acc[mt][nt][i];
      __syncthreads();
      const int r = 16 * mt + em, r2 = 16 * nt + en;
      if (r < b && r2 < b) {
        const float4 v = *reinterpret_cast<const float4 *>(so + e * 16 + 4 * quarter);
        *reinterpret_cast<float4 *>(partial + ((size_t)chunk * (b * b) + r * b + r2) * D + q0 + 4 * quarter) = v;
      }
      __syncthreads();
    }
}

template <int KT>
static void launch_dk_mfma(const float *X, const float *Gm, int64_t ld, int64_t n, int rows, int nchunks,
                           int D, int s, int b, float *partial, hipStream_t st) {
  const int gx = D / 16;
  const int64_t total = (int64_t)gx * nchunks;
  const int paired = (gx % 2 == 0) && (total % 16 == 0);
  hipLaunchKernelGGL((harp_grad_dk_mfma_kernel<KT>), dim3((unsigned)total), dim3(1024), 0, st, X, Gm, ld, n,
                     rows, D, s, b, gx, paired, partial);
}

static bool dk_mfma_supported(int b, int s, int D, const void *X, const void *Gm, int64_t ld,
                              const void *partial, int64_t nchunks) {
  if (b < 9 || b > 64 || s % 16 != 0 || D % 16 != 0) return false;
  if (ld % 4 != 0 || ld >= ((int64_t)1 << 26)) return false;
  if ((uintptr_t)X % 16 || (uintptr_t)Gm % 16 || (uintptr_t)partial % 16) return false;
  return (int64_t)(D / 16) * nchunks <= 0x7fffffff;
}

// the instantiation whose BMAX covers radix b
#define HARP_GRAD_BIG(b, CALL)            \
  do {                                    \
    if ((b) <= 16) { CALL(16); }          \
    else if ((b) <= 32) { CALL(32); }     \
    else if ((b) <= 48) { CALL(48); }     \
    else { CALL(64); }                    \
  } while (0)

// Run of K radix-2 stages with strides s, 2s, .., 2^(K-1) s.  Item q = hi s + lo owns the
// coordinates base + e s, e < 2^K, base = hi 2^K s + lo.  Stage i pairs e0 (bit i clear) with
// e0 + 2^i; that pair is block c = (i0 / (2 s_i)) s_i + i0 % s_i of the stage, i0 = base + e0 s,
// s_i = 2^i s.
struct GradRun {
  const float *blocks[3];
};

template <int K>
__device__ __forceinline__ void grad_run_blocks(const GradRun &run, int base, int s, int D,
                                                float (&kv)[K][1 << (K - 1)][4],
                                                int (&cidx)[K][1 << (K - 1)]) {
#pragma unroll
  for (int i = 0; i < K; ++i) {
    const int si = s << i;
#pragma unroll
    for (int p = 0; p < (1 << (K - 1)); ++p) {
      const int eh = p >> i, el = p & ((1 << i) - 1);
      const int e0 = (eh << (i + 1)) | el;
      const int i0 = base + e0 * s;
      const int c = (i0 / (2 * si)) * si + i0 % si;
      cidx[i][p] = c;
      const float4 f = *reinterpret_cast<const float4 *>(run.blocks[i] + (size_t)c * 4);
      kv[i][p][0] = f.x; kv[i][p][1] = f.y; kv[i][p][2] = f.z; kv[i][p][3] = f.w;
    }
  }
  (void)D;
}

// The E coordinates x[e s] of an item, float32 or bf16 (the caller's own rows in the first and
// last run, so that no separate conversion pass is needed); vec: stride 1 and aligned rows, the
// item is contiguous and moves with 16-byte accesses.
template <int E, typename T>
__device__ __forceinline__ void grad_load_item(const T *x, int s, bool vec, float (&v)[E]) {
  if (vec) {
    if constexpr (sizeof(T) == 4) {
#pragma unroll
      for (int q = 0; q < E / 4; ++q) {
        const float4 f = *reinterpret_cast<const float4 *>(x + 4 * q);
        v[4 * q] = f.x; v[4 * q + 1] = f.y; v[4 * q + 2] = f.z; v[4 * q + 3] = f.w;
      }
    } else if constexpr (E == 8) {
      const uint4 r = *reinterpret_cast<const uint4 *>(x);
      const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
      }
    } else {
      const uint2 r = *reinterpret_cast<const uint2 *>(x);
      v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
      v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
    }
  } else {
#pragma unroll
    for (int e = 0; e < E; ++e) v[e] = grad_widen(x[(size_t)e * s]);
  }
}
template <int E, typename T>
__device__ __forceinline__ void grad_store_item(T *y, int s, bool vec, const float (&v)[E]) {
  if (vec) {
    if constexpr (sizeof(T) == 4) {
#pragma unroll
      for (int q = 0; q < E / 4; ++q)
        *reinterpret_cast<float4 *>(y + 4 * q) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    } else {
      uint16_t h[E];
#pragma unroll
      for (int e = 0; e < E; ++e) grad_narrow(v[e], &h[e]);
      if constexpr (E == 8)
        *reinterpret_cast<uint4 *>(y) = make_uint4(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16),
                                                    h[4] | ((uint32_t)h[5] << 16), h[6] | ((uint32_t)h[7] << 16));
      else
        *reinterpret_cast<uint2 *>(y) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
    }
  } else {
#pragma unroll
    for (int e = 0; e < E; ++e) grad_narrow(v[e], y + (size_t)e * s);
  }
}

// TX: element type of the run's input rows (leading dimension ldx)
template <int K, typename TX = float>
__global__ __launch_bounds__(kGradThreads) void harp_grad_fwd_run_kernel(
    const TX *__restrict__ X, int64_t ldx, float *__restrict__ Y, int64_t ld, int64_t n, int rows,
    GradRun run, int nitems, int s, int aligned) {
  constexpr int E = 1 << K, H = E / 2;
  const int q = blockIdx.x * kGradThreads + threadIdx.x;
  if (q >= nitems) return;
  const int base = (q / s) * E * s + q % s;
  float kv[K][H][4];
  int cidx[K][H];
  grad_run_blocks<K>(run, base, s, 0, kv, cidx);
  const int64_t r0 = (int64_t)blockIdx.y * rows;
  const int64_t r1 = (r0 + rows < n) ? r0 + rows : n;
  // the next row is requested before the work on the current one
  // stride 1: the item's coordinates are contiguous (16-byte accesses when the row allows it)
  const bool vec = aligned && (s == 1) && (E % 4 == 0) && (ld % 4 == 0);
  const bool vecx = vec && ldx % (16 / (int)sizeof(TX)) == 0 && (uintptr_t)X % 16 == 0;
  auto load_item = [&](const TX *x, float (&v)[E]) { grad_load_item<E, TX>(x, s, vecx, v); };
  float nx[E];
#pragma unroll
  for (int e = 0; e < E; ++e) nx[e] = 0.f;
  if (r0 < r1) load_item(X + r0 * ldx + base, nx);
  for (int64_t row = r0; row < r1; ++row) {
    float *y = Y + row * ld + base;
    float v[E];
#pragma unroll
    for (int e = 0; e < E; ++e) v[e] = nx[e];
    if (row + 1 < r1) load_item(X + (row + 1) * ldx + base, nx);
#pragma unroll
    for (int i = 0; i < K; ++i)
#pragma unroll
      for (int p = 0; p < H; ++p) {
        const int eh = p >> i, el = p & ((1 << i) - 1);
        const int e0 = (eh << (i + 1)) | el, e1 = e0 | (1 << i);
        const float a = v[e0], b = v[e1];
        v[e0] = fmaf(b, kv[i][p][2], a * kv[i][p][0]);
        v[e1] = fmaf(b, kv[i][p][3], a * kv[i][p][1]);
      }
    if (vec) {
#pragma unroll
      for (int q = 0; q < E / 4; ++q)
        *reinterpret_cast<float4 *>(y + 4 * q) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    } else {
#pragma unroll
      for (int e = 0; e < E; ++e) y[(size_t)e * s] = v[e];
    }
  }
}

// partial sums of sub-stage i go to partial[i * pstride + (chunk * 4 + v) * D + c], D = d / 2
// TX: element type of the run's input rows X; the gradient is read from Gin (TGI) and the
// gradient passed back is written to Gout (TGO): the same float32 matrix in place, or the
// caller's G on the way in (last run) and the caller's dX on the way out (first run).  A thread
// reads its item of a row before it writes it, and no other thread touches that item.
template <int K, typename TX = float, typename TGI = float, typename TGO = float>
__global__ __launch_bounds__(kGradThreads) void harp_grad_bwd_run_kernel(
    const TX *__restrict__ X, int64_t ldx, const TGI *Gin, int64_t ldgi, TGO *Gout, int64_t ldgo,
    int64_t ld, int64_t n, int rows, GradRun run, int nitems, int s, int D,
    float *__restrict__ partial, size_t pstride, int aligned) {
  constexpr int E = 1 << K, H = E / 2;
  const int q = blockIdx.x * kGradThreads + threadIdx.x;
  if (q >= nitems) return;
  const int base = (q / s) * E * s + q % s;
  float kv[K][H][4], acc[K][H][4];
  int cidx[K][H];
  grad_run_blocks<K>(run, base, s, D, kv, cidx);
#pragma unroll
  for (int i = 0; i < K; ++i)
#pragma unroll
    for (int p = 0; p < H; ++p)
#pragma unroll
      for (int w = 0; w < 4; ++w) acc[i][p][w] = 0.f;
  const int64_t r0 = (int64_t)blockIdx.y * rows;
  const int64_t r1 = (r0 + rows < n) ? r0 + rows : n;
  const bool vec = aligned && (s == 1) && (E % 4 == 0) && (ld % 4 == 0);
  const bool vecx = vec && ldx % (16 / (int)sizeof(TX)) == 0 && (uintptr_t)X % 16 == 0;
  const bool vecgi = vec && ldgi % (16 / (int)sizeof(TGI)) == 0 && (uintptr_t)Gin % 16 == 0;
  const bool vecgo = vec && ldgo % (16 / (int)sizeof(TGO)) == 0 && (uintptr_t)Gout % 16 == 0;
  float nx[E], ng[E];
#pragma unroll
  for (int e = 0; e < E; ++e) nx[e] = ng[e] = 0.f;
  if (r0 < r1) {
    grad_load_item<E, TX>(X + r0 * ldx + base, s, vecx, nx);
    grad_load_item<E, TGI>(Gin + r0 * ldgi + base, s, vecgi, ng);
  }
  for (int64_t row = r0; row < r1; ++row) {
    TGO *g = Gout + row * ldgo + base;
    float xs[K][E], gv[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
      xs[0][e] = nx[e];
      gv[e] = ng[e];
    }
    if (row + 1 < r1) {   // the next row (its g is not written by anyone before this thread does)
      grad_load_item<E, TX>(X + (row + 1) * ldx + base, s, vecx, nx);
      grad_load_item<E, TGI>(Gin + (row + 1) * ldgi + base, s, vecgi, ng);
    }
    // inputs of the inner stages, recomputed
#pragma unroll
    for (int i = 0; i + 1 < K; ++i) {
#pragma unroll
      for (int p = 0; p < H; ++p) {
        const int eh = p >> i, el = p & ((1 << i) - 1);
        const int e0 = (eh << (i + 1)) | el, e1 = e0 | (1 << i);
        const float a = xs[i][e0], b = xs[i][e1];
        xs[i + 1][e0] = fmaf(b, kv[i][p][2], a * kv[i][p][0]);
        xs[i + 1][e1] = fmaf(b, kv[i][p][3], a * kv[i][p][1]);
      }
    }
#pragma unroll
    for (int i = K - 1; i >= 0; --i) {
#pragma unroll
      for (int p = 0; p < H; ++p) {
        const int eh = p >> i, el = p & ((1 << i) - 1);
        const int e0 = (eh << (i + 1)) | el, e1 = e0 | (1 << i);
        const float x0 = xs[i][e0], x1 = xs[i][e1], g0 = gv[e0], g1 = gv[e1];
        acc[i][p][0] = fmaf(x0, g0, acc[i][p][0]);
        acc[i][p][1] = fmaf(x0, g1, acc[i][p][1]);
        acc[i][p][2] = fmaf(x1, g0, acc[i][p][2]);
        acc[i][p][3] = fmaf(x1, g1, acc[i][p][3]);
        gv[e0] = fmaf(g1, kv[i][p][1], g0 * kv[i][p][0]);   // g K^T, row 0: k00 g0 + k01 g1
        gv[e1] = fmaf(g1, kv[i][p][3], g0 * kv[i][p][2]);
      }
    }
    grad_store_item<E, TGO>(g, s, vecgo, gv);
  }
#pragma unroll
  for (int i = 0; i < K; ++i)
#pragma unroll
    for (int p = 0; p < H; ++p)
#pragma unroll
      for (int w = 0; w < 4; ++w)
        partial[(size_t)i * pstride + ((size_t)blockIdx.y * 4 + w) * D + cidx[i][p]] = acc[i][p][w];
}

// dK[c][v] = sum over the chunks of partial[(chunk * BB + v) * D + c], in a fixed order: eight
// threads per value each add a contiguous eighth of the chunks (ascending), then the eight
// sums are added in ascending order.  For stage 0 the image holds diag(sigma) K_0, so row r of
// its gradient takes the sign of coordinate c b + r.
// blockIdx.y = sub-stage of a run (its partial sums start pstride floats further on).
struct GradReduceOut {
  float *dK[3];
  const int8_t *signs[3];
};
__global__ __launch_bounds__(kGradThreads) void harp_grad_reduce_kernel(
    const float *__restrict__ partial_all, size_t pstride, int nchunks, int D, int b,
    GradReduceOut out) {
  __shared__ float part[8][32];
  const float *__restrict__ partial = partial_all + (size_t)blockIdx.y * pstride;
  const int8_t *__restrict__ signs = out.signs[blockIdx.y];
  float *__restrict__ dK = out.dK[blockIdx.y];
  const int bb = b * b;
  const int64_t total = (int64_t)D * bb;
  const int lane = threadIdx.x & 31, slice = threadIdx.x >> 5;
  const int per = (nchunks + 7) / 8;
  const int k0 = slice * per, k1 = (k0 + per < nchunks) ? k0 + per : nchunks;
  const size_t step = (size_t)bb * D;
  for (int64_t i0 = (int64_t)blockIdx.x * 32; i0 < total; i0 += (int64_t)gridDim.x * 32) {
    const int64_t i = i0 + lane;
    const int v = (int)(i / D), c = (int)(i % D);     // consecutive lanes: consecutive c
    float sum = 0.f;
    if (i < total) {
      const float *p = partial + (size_t)v * D + c;
      int k = k0;
      for (; k + 8 <= k1; k += 8) {
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = p[(size_t)(k + u) * step];
#pragma unroll
        for (int u = 0; u < 8; ++u) sum += t[u];
      }
      for (; k < k1; ++k) sum += p[(size_t)k * step];
    }
    part[slice][lane] = sum;
    __syncthreads();
    if (slice == 0 && i < total) {
      float tot = part[0][lane];
#pragma unroll
      for (int u = 1; u < 8; ++u) tot += part[u][lane];
      if (signs) tot *= (float)signs[(size_t)c * b + v / b];
      dK[(size_t)c * bb + v] = tot;
    }
    __syncthreads();
  }
}

template <int B>
void launch_fwd(const float *X, float *Y, int64_t ld, int64_t n, int rows, int nchunks,
                const float *blocks, int D, int s, hipStream_t st) {
  hipLaunchKernelGGL((harp_grad_fwd_kernel<B>), dim3((D + kGradThreads - 1) / kGradThreads, nchunks),
                     dim3(kGradThreads), 0, st, X, Y, ld, n, rows, blocks, D, s);
}
template <int B>
void launch_bwd(const float *X, float *G, int64_t ld, int64_t n, int rows, int nchunks,
                const float *blocks, int D, int s, float *partial, hipStream_t st) {
  hipLaunchKernelGGL((harp_grad_bwd_kernel<B>), dim3((D + kGradThreads - 1) / kGradThreads, nchunks),
                     dim3(kGradThreads), 0, st, X, G, ld, n, rows, blocks, D, s, partial);
}

#define HARP_GRAD_SWITCH(b, CALL)  \
  switch (b) {                     \
    case 2: CALL(2); break;        \
    case 3: CALL(3); break;        \
    case 4: CALL(4); break;        \
    case 5: CALL(5); break;        \
    case 6: CALL(6); break;        \
    case 7: CALL(7); break;        \
    default: CALL(8); break;       \
  }

template <typename TS, typename TD>
void launch_convert(const TS *src, int64_t lds_, TD *dst, int64_t ldd, int64_t n, int64_t d,
                    hipStream_t st) {
  const bool vec = (d % 8 == 0) && (lds_ % 8 == 0) && (ldd % 8 == 0) && ((uintptr_t)src % 16 == 0) &&
                   ((uintptr_t)dst % 16 == 0);
  const int64_t per = vec ? 8 * kGradThreads : kGradThreads;
  // the row index is blockIdx.y (at most 65535 per launch)
  for (int64_t r0 = 0; r0 < n; r0 += 65535) {
    const int64_t nr = std::min<int64_t>(65535, n - r0);
    const unsigned gx = (unsigned)std::min<int64_t>((d + per - 1) / per, 64);
    if (vec)
      hipLaunchKernelGGL((harp_grad_convert_kernel<TS, TD, true>), dim3(gx, (unsigned)nr),
                         dim3(kGradThreads), 0, st, src + r0 * lds_, lds_, dst + r0 * ldd, ldd, nr, (int)d);
    else
      hipLaunchKernelGGL((harp_grad_convert_kernel<TS, TD, false>), dim3(gx, (unsigned)nr),
                         dim3(kGradThreads), 0, st, src + r0 * lds_, lds_, dst + r0 * ldd, ldd, nr, (int)d);
  }
}

}  // namespace

// Row chunks per launch: a fused run of three stages has only d / 8 threads per row, so the
// rows have to supply the parallelism (d = 4096: 2 workgroups x 256 chunks).
int grad_chunks(int64_t n) {
  const int64_t c = (n + 7) / 8;
  return (int)std::max<int64_t>(1, std::min<int64_t>(c, 256));
}

// Segments of the backward pass: runs of up to three radix-2 stages, single stages otherwise.
struct GradSegment {
  int t0, k;
};
static std::vector<GradSegment> grad_segments(const harp_plan *plan) {
  std::vector<GradSegment> seg;
  const int m = plan->m;
  int t = 0;
  while (t < m) {
    int k = 1;
    if (plan->radices[t] == 2)
      while (k < 3 && t + k < m && plan->radices[t + k] == 2) ++k;
    seg.push_back(GradSegment{t, k});
    t += k;
  }
  return seg;
}

// Stages of radix above 8 take longer row chunks: blockIdx.z already supplies parallelism, and a
// chunk costs one read of the block column per thread and b * b partial sums per block.
static int grad_big_rows(int64_t n) {
  const int nchunks = grad_chunks(n);
  return std::max((int)((n + nchunks - 1) / nchunks), 64);
}
static int grad_big_chunks(int64_t n) {
  const int rb = grad_big_rows(n);
  return (int)std::max<int64_t>(1, (n + rb - 1) / rb);
}

size_t grad_workspace_bytes(const harp_plan *plan, int64_t n) {
  int bsmall = 6;   // a run of three radix-2 stages leaves 3 * (d / 2) * 4 partial values per chunk
  int bbig = 0;
  for (int32_t b : plan->radices) (b > 8 ? bbig : bsmall) = std::max(b > 8 ? bbig : bsmall, (int)b);
  const size_t mat = (size_t)n * (size_t)plan->d * 4;
  const size_t nseg = grad_segments(plan).size();
  const size_t partial = std::max((size_t)grad_chunks(n) * bsmall, (size_t)grad_big_chunks(n) * bbig) *
                         (size_t)plan->d * 4;
  // a stage of radix above 8 passes the gradient back out of place: one more matrix
  return (nseg + 1 + (bbig > 0 ? 1 : 0)) * mat + partial;
}

harp_status_t launch_grad(const harp_plan *plan, const void *X, int64_t ldx, const void *G,
                          int64_t ldg, int64_t n, harp_dtype_t dt, float *const *dK, void *dX,
                          int64_t lddx, void *ws, hipStream_t st) {
  const std::vector<ColStage> &stages = plan->col[DIR_FWD];
  const std::vector<GradSegment> seg = grad_segments(plan);
  const int nseg = (int)seg.size();
  const int64_t d = plan->d;
  const int nchunks = grad_chunks(n);
  const int rows = (int)((n + nchunks - 1) / nchunks);
  const int rows_big = grad_big_rows(n);
  const int nchunks_big = grad_big_chunks(n);
  const size_t mat = (size_t)n * (size_t)d;
  int bmax = 0;
  for (int32_t b : plan->radices) bmax = std::max(bmax, (int)b);
  float *act = (float *)ws;                 // act[i] = input of segment i
  float *g = act + (size_t)nseg * mat;      // gradient, updated in place (radix <= 8) ...
  float *g2 = g + mat;                      // ... or into the other of two matrices (radix >= 9)
  float *partial = g + (bmax > 8 ? 2 : 1) * mat;
  const size_t pstride = (size_t)nchunks * 4 * (size_t)(d / 2);   // one radix-2 stage's partials
  // 16-byte accesses of the stride-1 runs need the float32 copies on 16-byte boundaries
  const int aligned = ((uintptr_t)ws % 16 == 0) && (mat % 4 == 0);
  auto run_of = [&](const GradSegment &sg) {
    GradRun run;
    for (int i = 0; i < 3; ++i) run.blocks[i] = stages[sg.t0 + std::min(i, sg.k - 1)].blocks;
    return run;
  };
  // A run of radix-2 stages at the start reads the caller's X itself (forward and backward), one
  // at the end reads the caller's G, and the first run writes dX: no separate conversion pass.
  const bool bf = (dt == HARP_BF16);
  const bool first_run = seg[0].k > 1, last_run = seg[nseg - 1].k > 1;
  const bool dx_direct = first_run && dX != nullptr;
  if (n > 0) {
    if (!first_run) {
      if (bf) launch_convert((const uint16_t *)X, ldx, act, d, n, d, st);
      else launch_convert((const float *)X, ldx, act, d, n, d, st);
    }
    if (!last_run) {
      if (bf) launch_convert((const uint16_t *)G, ldg, g, d, n, d, st);
      else launch_convert((const float *)G, ldg, g, d, n, d, st);
    }
    for (int i = 0; i + 1 < nseg; ++i) {
      const ColStage &cs = stages[seg[i].t0];
      const float *in = act + (size_t)i * mat;
      float *out = act + (size_t)(i + 1) * mat;
      if (seg[i].k > 1) {
        const int nitems = (int)(d >> seg[i].k);
        const dim3 grid((nitems + kGradThreads - 1) / kGradThreads, nchunks);
#define HARP_GRAD_FWD_RUN(KK)                                                                       \
  do {                                                                                              \
    if (i == 0 && bf)                                                                               \
      hipLaunchKernelGGL((harp_grad_fwd_run_kernel<KK, uint16_t>), grid, dim3(kGradThreads), 0, st, \
                         (const uint16_t *)X, ldx, out, d, n, rows, run_of(seg[i]), nitems, cs.s,   \
                         aligned);                                                                  \
    else if (i == 0)                                                                                \
      hipLaunchKernelGGL((harp_grad_fwd_run_kernel<KK, float>), grid, dim3(kGradThreads), 0, st,    \
                         (const float *)X, ldx, out, d, n, rows, run_of(seg[i]), nitems, cs.s,      \
                         aligned);                                                                  \
    else                                                                                            \
      hipLaunchKernelGGL((harp_grad_fwd_run_kernel<KK, float>), grid, dim3(kGradThreads), 0, st,    \
                         in, d, out, d, n, rows, run_of(seg[i]), nitems, cs.s, aligned);            \
  } while (0)
        if (seg[i].k == 3) HARP_GRAD_FWD_RUN(3);
        else HARP_GRAD_FWD_RUN(2);
#undef HARP_GRAD_FWD_RUN
      } else if (cs.b > 8 && mfma_pass_supported(plan->grad_mfma[0][seg[i].t0], in, d, out, d)) {
        // the stage on the matrix cores (float32 operands), as in a split program
        if (launch_mfma_pass(plan, plan->grad_mfma[0][seg[i].t0], in, d, HARP_F32, out, d, HARP_F32, n,
                             false, st) != HARP_OK)
          return HARP_ERR_DEVICE;
      } else if (cs.b > 8) {
        const int D = (int)(d / cs.b);
#define HARP_GRAD_BIG_FWD(BM)                                                                     \
  hipLaunchKernelGGL((harp_grad_apply_big_kernel<BM, false>),                                     \
                     dim3((D + 63) / 64, nchunks_big, (cs.b + 3) / 4), dim3(kGradThreads), 0, st, \
                     in, out, d, n, rows_big, cs.blocks, D, cs.s, cs.b)
        HARP_GRAD_BIG(cs.b, HARP_GRAD_BIG_FWD);
#undef HARP_GRAD_BIG_FWD
      } else {
        const int D = (int)(d / cs.b);
#define HARP_GRAD_FWD(BB) launch_fwd<BB>(in, out, d, n, rows, nchunks, cs.blocks, D, cs.s, st)
        HARP_GRAD_SWITCH(cs.b, HARP_GRAD_FWD)
#undef HARP_GRAD_FWD
      }
    }
  }
  for (int i = nseg - 1; i >= 0; --i) {
    const ColStage &cs = stages[seg[i].t0];
    const float *in = act + (size_t)i * mat;
    if (n > 0) {
      if (seg[i].k > 1) {
        const int nitems = (int)(d >> seg[i].k);
        const dim3 grid((nitems + kGradThreads - 1) / kGradThreads, nchunks);
        // what this run reads and writes: the caller's rows at either end, float32 copies between
        const bool xc = (i == 0), gic = (i == nseg - 1), goc = (i == 0) && dx_direct;
#define HARP_GRAD_BWD_RUN(KK, TX_, TGI_, TGO_)                                                       \
  hipLaunchKernelGGL((harp_grad_bwd_run_kernel<KK, TX_, TGI_, TGO_>), grid, dim3(kGradThreads), 0,   \
                     st, xc ? (const TX_ *)X : (const TX_ *)in, xc ? ldx : d,                        \
                     gic ? (const TGI_ *)G : (const TGI_ *)g, gic ? ldg : d,                         \
                     goc ? (TGO_ *)dX : (TGO_ *)g, goc ? lddx : d, d, n, rows, run_of(seg[i]),      \
                     nitems, cs.s, (int)(d / 2), partial, pstride, aligned)
#define HARP_GRAD_BWD_TYPES(KK)                                                          \
  do {                                                                                   \
    if (!bf) HARP_GRAD_BWD_RUN(KK, float, float, float);                                 \
    else if (xc && gic && goc) HARP_GRAD_BWD_RUN(KK, uint16_t, uint16_t, uint16_t);      \
    else if (xc && gic) HARP_GRAD_BWD_RUN(KK, uint16_t, uint16_t, float);                \
    else if (xc && goc) HARP_GRAD_BWD_RUN(KK, uint16_t, float, uint16_t);                \
    else if (xc) HARP_GRAD_BWD_RUN(KK, uint16_t, float, float);                          \
    else if (gic) HARP_GRAD_BWD_RUN(KK, float, uint16_t, float);                         \
    else HARP_GRAD_BWD_RUN(KK, float, float, float);                                     \
  } while (0)
        if (seg[i].k == 3) HARP_GRAD_BWD_TYPES(3);
        else HARP_GRAD_BWD_TYPES(2);
#undef HARP_GRAD_BWD_TYPES
#undef HARP_GRAD_BWD_RUN
      } else if (cs.b > 8) {
        const int D = (int)(d / cs.b);
        const dim3 grid((D + 63) / 64, nchunks_big, (cs.b + 3) / 4);
        // gradient passed back: the transposed blocks on the matrix cores where the stage allows
        const bool mf = mfma_pass_supported(plan->grad_mfma[1][seg[i].t0], g, d, g2, d);
        const bool dkm = dk_mfma_supported(cs.b, cs.s, D, in, g, d, partial, nchunks_big);
        if (dkm) {
          switch ((cs.b + 15) / 16) {
            case 1: launch_dk_mfma<1>(in, g, d, n, rows_big, nchunks_big, D, cs.s, cs.b, partial, st); break;
            case 2: launch_dk_mfma<2>(in, g, d, n, rows_big, nchunks_big, D, cs.s, cs.b, partial, st); break;
            case 3: launch_dk_mfma<3>(in, g, d, n, rows_big, nchunks_big, D, cs.s, cs.b, partial, st); break;
            default: launch_dk_mfma<4>(in, g, d, n, rows_big, nchunks_big, D, cs.s, cs.b, partial, st); break;
          }
        }
#define HARP_GRAD_BIG_BWD(BM)                                                                      \
  if (!dkm)                                                                                        \
    hipLaunchKernelGGL((harp_grad_dk_big_kernel<BM>), grid, dim3(kGradThreads), 0, st, in, g, d, n, \
                       rows_big, D, cs.s, cs.b, partial);                                          \
  if (!mf)                                                                                         \
    hipLaunchKernelGGL((harp_grad_apply_big_kernel<BM, true>), grid, dim3(kGradThreads), 0, st, g, \
                       g2, d, n, rows_big, cs.blocks, D, cs.s, cs.b)
        HARP_GRAD_BIG(cs.b, HARP_GRAD_BIG_BWD);
#undef HARP_GRAD_BIG_BWD
        if (mf && launch_mfma_pass(plan, plan->grad_mfma[1][seg[i].t0], g, d, HARP_F32, g2, d, HARP_F32, n,
                                   false, st) != HARP_OK)
          return HARP_ERR_DEVICE;
        std::swap(g, g2);
      } else {
        const int D = (int)(d / cs.b);
#define HARP_GRAD_BWD(BB) launch_bwd<BB>(in, g, d, n, rows, nchunks, cs.blocks, D, cs.s, partial, st)
        HARP_GRAD_SWITCH(cs.b, HARP_GRAD_BWD)
#undef HARP_GRAD_BWD
      }
    }
    // the run's sub-stages in one reduction launch
    {
      const int b = stages[seg[i].t0].b;
      const int D = (int)(d / b);
      const int64_t total = (int64_t)D * b * b;
      const unsigned gx = (unsigned)std::min<int64_t>((total + 31) / 32, 8192);
      GradReduceOut ro{};
      for (int j = 0; j < seg[i].k; ++j) {
        ro.dK[j] = dK[seg[i].t0 + j];
        ro.signs[j] = (seg[i].t0 + j == 0) ? plan->dev_signs : nullptr;
      }
      hipLaunchKernelGGL(harp_grad_reduce_kernel, dim3(gx, (unsigned)seg[i].k), dim3(kGradThreads), 0, st,
                         partial, pstride, n > 0 ? (b > 8 ? nchunks_big : nchunks) : 0, D, b, ro);
    }
  }
  if (dX && n > 0 && !dx_direct) {
    if (bf) launch_convert(g, d, (uint16_t *)dX, lddx, n, d, st);
    else launch_convert(g, d, (float *)dX, lddx, n, d, st);
  }
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

}  // namespace harp
