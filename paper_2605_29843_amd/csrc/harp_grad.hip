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
// stay in registers.  Radices up to 8 (the plan's dense per-stage image with the signs folded
// into stage 0 is the one the column-mode passes use).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

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

// dst[r, c] = convert(src[r, c])
template <typename TS, typename TD>
__global__ __launch_bounds__(kGradThreads) void harp_grad_convert_kernel(
    const TS *__restrict__ src, int64_t lds_, TD *__restrict__ dst, int64_t ldd, int64_t n, int d) {
  const int64_t row = blockIdx.y;
  for (int c = blockIdx.x * kGradThreads + threadIdx.x; c < d; c += gridDim.x * kGradThreads)
    grad_narrow(grad_widen(src[row * lds_ + c]), dst + row * ldd + c);
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

// dK[c][v] = sum over chunks (ascending) of partial[(chunk * BB + v) * D + c]; for stage 0 the
// image holds diag(sigma) K_0, so row r of its gradient takes the sign of coordinate c b + r.
__global__ __launch_bounds__(kGradThreads) void harp_grad_reduce_kernel(
    const float *__restrict__ partial, int nchunks, int D, int b, const int8_t *__restrict__ signs,
    float *__restrict__ dK) {
  const int bb = b * b;
  const int64_t total = (int64_t)D * bb;
  for (int64_t i = (int64_t)blockIdx.x * kGradThreads + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kGradThreads) {
    const int v = (int)(i / D), c = (int)(i % D);     // consecutive threads: consecutive c
    // loads eight chunks ahead, additions in ascending chunk order
    const float *p = partial + (size_t)v * D + c;
    const size_t step = (size_t)bb * D;
    float sum = 0.f;
    int k = 0;
    for (; k + 8 <= nchunks; k += 8) {
      float t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = p[(size_t)(k + u) * step];
#pragma unroll
      for (int u = 0; u < 8; ++u) sum += t[u];
    }
    for (; k < nchunks; ++k) sum += p[(size_t)k * step];
    if (signs) sum *= (float)signs[(size_t)c * b + v / b];
    dK[(size_t)c * bb + v] = sum;
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
  // the row index is blockIdx.y (at most 65535 per launch)
  for (int64_t r0 = 0; r0 < n; r0 += 65535) {
    const int64_t nr = std::min<int64_t>(65535, n - r0);
    const unsigned gx = (unsigned)std::min<int64_t>((d + kGradThreads - 1) / kGradThreads, 64);
    hipLaunchKernelGGL((harp_grad_convert_kernel<TS, TD>), dim3(gx, (unsigned)nr), dim3(kGradThreads),
                       0, st, src + r0 * lds_, lds_, dst + r0 * ldd, ldd, nr, (int)d);
  }
}

}  // namespace

int grad_chunks(int64_t n) {
  const int64_t c = (n + 31) / 32;
  return (int)std::max<int64_t>(1, std::min<int64_t>(c, 128));
}

size_t grad_workspace_bytes(const harp_plan *plan, int64_t n) {
  int bmax = 2;
  for (int32_t b : plan->radices) bmax = std::max(bmax, (int)b);
  const size_t mat = (size_t)n * (size_t)plan->d * 4;
  return (size_t)(plan->m + 1) * mat + (size_t)grad_chunks(n) * (size_t)plan->d * bmax * 4;
}

harp_status_t launch_grad(const harp_plan *plan, const void *X, int64_t ldx, const void *G,
                          int64_t ldg, int64_t n, harp_dtype_t dt, float *const *dK, void *dX,
                          int64_t lddx, void *ws, hipStream_t st) {
  const std::vector<ColStage> &stages = plan->col[DIR_FWD];
  const int m = plan->m;
  const int64_t d = plan->d;
  const int nchunks = grad_chunks(n);
  const int rows = (int)((n + nchunks - 1) / nchunks);
  const size_t mat = (size_t)n * (size_t)d;
  float *act = (float *)ws;                 // act[t] = input of stage t, t < m
  float *g = act + (size_t)m * mat;         // gradient, updated in place
  float *partial = g + mat;
  if (n > 0) {
    if (dt == HARP_BF16) {
      launch_convert((const uint16_t *)X, ldx, act, d, n, d, st);
      launch_convert((const uint16_t *)G, ldg, g, d, n, d, st);
    } else {
      launch_convert((const float *)X, ldx, act, d, n, d, st);
      launch_convert((const float *)G, ldg, g, d, n, d, st);
    }
    for (int t = 0; t + 1 < m; ++t) {
      const ColStage &cs = stages[t];
      const int D = (int)(d / cs.b);
#define HARP_GRAD_FWD(BB) \
  launch_fwd<BB>(act + (size_t)t * mat, act + (size_t)(t + 1) * mat, d, n, rows, nchunks, cs.blocks, D, cs.s, st)
      HARP_GRAD_SWITCH(cs.b, HARP_GRAD_FWD)
#undef HARP_GRAD_FWD
    }
  }
  for (int t = m - 1; t >= 0; --t) {
    const ColStage &cs = stages[t];
    const int D = (int)(d / cs.b);
    if (n > 0) {
#define HARP_GRAD_BWD(BB) \
  launch_bwd<BB>(act + (size_t)t * mat, g, d, n, rows, nchunks, cs.blocks, D, cs.s, partial, st)
      HARP_GRAD_SWITCH(cs.b, HARP_GRAD_BWD)
#undef HARP_GRAD_BWD
    }
    const int64_t total = (int64_t)D * cs.b * cs.b;
    const unsigned gx = (unsigned)std::min<int64_t>((total + kGradThreads - 1) / kGradThreads, 4096);
    hipLaunchKernelGGL(harp_grad_reduce_kernel, dim3(gx), dim3(kGradThreads), 0, st, partial,
                       n > 0 ? nchunks : 0, D, cs.b, t == 0 ? plan->dev_signs : nullptr, dK[t]);
  }
  if (dX && n > 0) {
    if (dt == HARP_BF16) launch_convert(g, d, (uint16_t *)dX, lddx, n, d, st);
    else launch_convert(g, d, (float *)dX, lddx, n, d, st);
  }
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

}  // namespace harp
