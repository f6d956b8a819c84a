// Row-pipelined kernel for pure radix-2 chains of orthogonal blocks, d = 2^(K0+K1+K2) <= 4096,
// bf16 I/O.  Every stage but the last is executed as three lifting steps, the last as a dense
// 2x2 that also carries all pending signs (see the plan builder), so the inner loop is fused
// multiply-adds only.
//
// The 10..12 stages are cut into three passes of K0, K1, K2 consecutive stages.  A workgroup
// has three wave groups of d/16 threads; group g executes pass g and nothing else, so a thread
// keeps the rotation parameters of its own 16 coordinates x K stages in registers for the
// whole launch (they are read from device memory exactly once per workgroup), and rows flow
// through the groups like an assembly line:
//
//    step k:  group 0  takes row k (prefetched from device memory several rows ahead),
//                      applies pass 0, writes the row to LDS buffer A[k & 1]
//             group 1  reads row k-1 from A[(k-1) & 1], applies pass 1, writes B[k & 1]
//             group 2  reads row k-2 from B[(k-1) & 1], applies pass 2, rounds to bf16 and
//                      stores it to device memory
//             one workgroup barrier
//
// so loads, the three passes and stores of different rows overlap, and the three groups give
// every SIMD three independent instruction streams.  The stride permutations of Eq. (7)
// appear only as the LDS addresses a group reads and writes (Lemma 1 indexing); the LDS
// positions are swizzled so that the contiguous 16-float accesses of the stride-1 pass and
// the stride-16 / stride-256 accesses of the other passes are all free of bank conflicts.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "harp_internal.h"

namespace harp {

namespace {

constexpr int kPrefetch = 4;
// With READ_AHEAD groups 1 and 2 issue the LDS reads of their next row one step before they
// compute it (two more pipeline steps per tile).  Measured on MI355X it does not pay: LDS
// instructions and arithmetic of the waves of one SIMD overlap poorly either way, and tiles
// of 8 rows lose more to the longer fill and drain than they gain.
constexpr bool READ_AHEAD = false;

// LDS position (in floats) of logical coordinate i of a row: 16 floats of padding per 256,
// and the four 4-float chunks of every 16-float segment rotated by (segment / 2).
__device__ __forceinline__ int phys_index(int i) {
  return (i >> 8) * 272 + (i & 0xF0) + ((((i >> 2) + (i >> 5)) & 3) << 2) + (i & 3);
}

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  bf2 v;
  v.x = (__bf16)lo;
  v.y = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

// K radix-2 stages on SPT = 16 / 2^K sub-tensors held in x[16].  Stages are lifted rotations
// (x0 += a x1; x1 += b x0; x0 += a x1, values (a, b) at ((e * P/2 + p) * 2) of the
// sub-tensor's block of parameters); with LD the K-th stage is a dense 2x2 whose four values
// per pair follow the (K-1) * P lifted values.
template <int K, bool DESC, bool LD>
__device__ __forceinline__ void lift_stages(float (&x)[16], const float (&prm)[16 * (K + (LD ? 1 : 0))]) {
  constexpr int P = 1 << K, SPT = 16 / P, NV = (K + (LD ? 1 : 0)) * P;
#pragma unroll
  for (int u = 0; u < SPT; ++u) {
#pragma unroll
    for (int e = 0; e < K; ++e) {
      const int bp = DESC ? K - 1 - e : e;
#pragma unroll
      for (int p = 0; p < P / 2; ++p) {
        const int j0 = u * P + (((p >> bp) << (bp + 1)) | (p & ((1 << bp) - 1)));
        const int j1 = j0 | (1 << bp);
        float x0 = x[j0], x1 = x[j1];
        if (LD && e == K - 1) {
          const int v0 = u * NV + (K - 1) * P + p * 4;
          x[j0] = fmaf(x1, prm[v0 + 2], x0 * prm[v0 + 0]);
          x[j1] = fmaf(x1, prm[v0 + 3], x0 * prm[v0 + 1]);
        } else {
          const float a = prm[u * NV + (e * (P / 2) + p) * 2 + 0];
          const float b = prm[u * NV + (e * (P / 2) + p) * 2 + 1];
          x0 = fmaf(a, x1, x0);
          x1 = fmaf(b, x0, x1);
          x0 = fmaf(a, x1, x0);
          x[j0] = x0;
          x[j1] = x1;
        }
      }
    }
  }
}

// Body of one wave group.  ROLE 0 = first pass (reads device memory), 1 = middle, 2 = last
// (writes device memory; its K-th stage is the program's last and is dense).  LOGS = log2 of
// the stride of the pass's lowest digit; the pass with LOGS == 0 touches 16 contiguous
// coordinates per thread (16-byte vector accesses), the others touch single coordinates.
// Every group executes the same number of barriers (nr + 2, or nr + 4 with read-ahead).
template <int K, int LOGS, bool DESC, int ROLE, int D>
__device__ __forceinline__ void pipe_group(const PassDesc &pd, const int t, const float *rd_buf,
                                           float *wr_buf, const uint16_t *__restrict__ X,
                                           const int64_t ldx, uint16_t *__restrict__ Y,
                                           const int64_t ldy, const int nr) {
  constexpr bool LD = (ROLE == 2);
  constexpr int P = 1 << K, SPT = 16 / P, TG = D / 16, NV = (K + (LD ? 1 : 0)) * P;
  constexpr int ROWBUF = (D / 256) * 272;
  constexpr int S = 1 << LOGS;
  constexpr bool CONTIG = (LOGS == 0);
  constexpr int NRAW = CONTIG ? 8 : 16;            // dwords of raw input per row and thread
  constexpr int PF = CONTIG ? kPrefetch : kPrefetch - 1;
  const int nq = pd.nq;
  const float *__restrict__ params = pd.params;

  float prm[SPT * NV];
  unsigned base[SPT];
#pragma unroll
  for (int u = 0; u < SPT; ++u) {
    const unsigned q = (unsigned)t + u * TG;
#pragma unroll
    for (int v = 0; v < NV; ++v) prm[u * NV + v] = params[(unsigned)(v * nq) + q];
    const unsigned hi = q >> LOGS, lo = q & (S - 1);
    base[u] = ((hi << K) << LOGS) | lo;
  }
  // logical coordinate of element (u, j): base[u] | (j << LOGS) (the bit fields are disjoint)
  auto lds_off = [&](int e) -> int {
    const int u = e / P, j = e % P;
    return phys_index((int)(base[u] | ((unsigned)j << LOGS)));
  };
  auto glb_off = [&](int e) -> unsigned {   // element offset inside a row
    const int u = e / P, j = e % P;
    return base[u] | ((unsigned)j << LOGS);
  };

  // ---- ROLE 0: prefetch the first rows.  Contiguous side: 8 dwords of bf16 pairs per row;
  // strided side: one bf16 per dword (widened when consumed).
  uint32_t pre[PF][NRAW];
  auto issue_load = [&](int slot, int row) {
    const uint16_t *xr = X + (int64_t)row * ldx;   // wave-uniform
    if (CONTIG) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint4 v = *reinterpret_cast<const uint4 *>(xr + glb_off(8 * h));
        pre[slot][4 * h + 0] = v.x; pre[slot][4 * h + 1] = v.y;
        pre[slot][4 * h + 2] = v.z; pre[slot][4 * h + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) pre[slot][e % NRAW] = xr[glb_off(e)];
    }
  };
  if (ROLE == 0) {
#pragma unroll
    for (int s = 0; s < PF; ++s)
      if (s < nr) issue_load(s, s);
  }

  // The step loop is unrolled by UNR so that prefetch slots, buffer parities and the two
  // register sets of the optional LDS read-ahead are static.  Without read-ahead group g
  // reads and computes row k-g at step k (nr + 2 steps); with it group 1 reads row k-1 and
  // computes row k-2, group 2 reads row k-3 and computes row k-4 (nr + 4 steps).  One barrier
  // per step.
  constexpr int UNR = (ROLE == 0) ? (PF % 2 ? 2 * PF : PF) : 2;
  constexpr int RD_LAG = READ_AHEAD ? ((ROLE == 0) ? 0 : (ROLE == 1 ? 1 : 3)) : ROLE;
  const int nsteps = nr + (READ_AHEAD ? 4 : 2);
  float xa[16], xb[16];
  for (int k0 = 0; k0 < nsteps; k0 += UNR) {
#pragma unroll
    for (int s = 0; s < UNR; ++s) {
      const int k = k0 + s;
      if (k >= nsteps) break;
      float(&xn)[16] = (s & 1) ? xb : xa;   // filled in this step
      float(&xc)[16] = (ROLE == 0 || !READ_AHEAD) ? xn : ((s & 1) ? xa : xb);   // computed now
      const int r_rd = k - RD_LAG;
      const int r_cp = (ROLE == 0 || !READ_AHEAD) ? r_rd : r_rd - 1;
      if (r_rd >= 0 && r_rd < nr) {
        if (ROLE == 0) {
          const int slot = s % PF;
          if (CONTIG) {
#pragma unroll
            for (int m = 0; m < 8; ++m) {
              const uint32_t w = pre[slot][m % NRAW];
              xn[2 * m] = __uint_as_float(w << 16);
              xn[2 * m + 1] = __uint_as_float(w & 0xffff0000u);
            }
          } else {
#pragma unroll
            for (int e = 0; e < 16; ++e) xn[e] = __uint_as_float(pre[slot][e % NRAW] << 16);
          }
          if (r_rd + PF < nr) issue_load(slot, r_rd + PF);
        } else {
          const float *b = rd_buf + ((s + 1) & 1) * ROWBUF;   // written in step k - 1
          if (CONTIG) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              const float4 f = *reinterpret_cast<const float4 *>(b + lds_off(4 * c));
              xn[4 * c] = f.x; xn[4 * c + 1] = f.y; xn[4 * c + 2] = f.z; xn[4 * c + 3] = f.w;
            }
          } else {
#pragma unroll
            for (int e = 0; e < 16; ++e) xn[e] = b[lds_off(e)];
          }
        }
      }
      if (r_cp >= 0 && r_cp < nr) {
        lift_stages<K, DESC, LD>(xc, prm);
        if (ROLE == 2) {
          uint16_t *yr = Y + (int64_t)r_cp * ldy;   // wave-uniform
          if (CONTIG) {
            uint32_t w[8];
#pragma unroll
            for (int m = 0; m < 8; ++m) w[m] = cvt_pk_bf16(xc[2 * m], xc[2 * m + 1]);
#pragma unroll
            for (int h = 0; h < 2; ++h)
              *reinterpret_cast<uint4 *>(yr + glb_off(8 * h)) =
                  make_uint4(w[4 * h], w[4 * h + 1], w[4 * h + 2], w[4 * h + 3]);
          } else {
#pragma unroll
            for (int m = 0; m < 8; ++m) {
              const uint32_t w = cvt_pk_bf16(xc[2 * m], xc[2 * m + 1]);
              yr[glb_off(2 * m)] = (uint16_t)(w & 0xffffu);
              yr[glb_off(2 * m + 1)] = (uint16_t)(w >> 16);
            }
          }
        } else {
          float *b = wr_buf + (s & 1) * ROWBUF;               // read by the next group in step k + 1
          if (CONTIG) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
              *reinterpret_cast<float4 *>(b + lds_off(4 * c)) =
                  make_float4(xc[4 * c], xc[4 * c + 1], xc[4 * c + 2], xc[4 * c + 3]);
          } else {
#pragma unroll
            for (int e = 0; e < 16; ++e) b[lds_off(e)] = xc[e];
          }
        }
      }
      __syncthreads();
    }
  }
}

template <int K0, int K1, int K2, bool TRN>
__global__ __launch_bounds__(3 << (K0 + K1 + K2 - 4)) void harp_pipe_bf16_kernel(
    const uint16_t *__restrict__ X, int64_t ldx, uint16_t *__restrict__ Y, int64_t ldy, int64_t n,
    int R, const Program *__restrict__ progp) {
  constexpr int D = 1 << (K0 + K1 + K2), TG = D / 16, ROWBUF = (D / 256) * 272;
  __shared__ float bufA[2 * ROWBUF];
  __shared__ float bufB[2 * ROWBUF];
  const int g = __builtin_amdgcn_readfirstlane((int)threadIdx.x / TG);  // wave-uniform
  const int t = (int)threadIdx.x % TG;
  const int64_t row0 = (int64_t)blockIdx.x * R;
  const int nr = (int)((n - row0 < R) ? (n - row0) : R);
  const Program &prog = *progp;
  const uint16_t *Xt = X + row0 * ldx;
  uint16_t *Yt = Y + row0 * ldy;
  // stride of each pass's lowest digit: ascending for apply, descending for apply_transpose
  constexpr int LS0 = TRN ? K1 + K2 : 0, LS1 = TRN ? K2 : K0, LS2 = TRN ? 0 : K0 + K1;
  if (g == 0)
    pipe_group<K0, LS0, TRN, 0, D>(prog.pass[0], t, nullptr, bufA, Xt, ldx, Yt, ldy, nr);
  else if (g == 1)
    pipe_group<K1, LS1, TRN, 1, D>(prog.pass[1], t, bufA, bufB, Xt, ldx, Yt, ldy, nr);
  else
    pipe_group<K2, LS2, TRN, 2, D>(prog.pass[2], t, bufB, nullptr, Xt, ldx, Yt, ldy, nr);
}

template <int K0, int K1, int K2, bool TRN>
harp_status_t launch_pipe_inst(const Program *dprog, const void *X, int64_t ldx, void *Y,
                               int64_t ldy, int64_t n, int R, hipStream_t stream) {
  constexpr int NT = 3 << (K0 + K1 + K2 - 4);
  const int64_t tiles = (n + R - 1) / R;
  if (tiles > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((harp_pipe_bf16_kernel<K0, K1, K2, TRN>), dim3((unsigned)tiles), dim3(NT), 0,
                     stream, (const uint16_t *)X, ldx, (uint16_t *)Y, ldy, n, R, dprog);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

}  // namespace

// True when the program is three rotation passes on a power-of-two d that this file has an
// instantiation for, and the buffers allow 16-byte row accesses.
bool pipe_supported(const harp_plan *plan, const Program &hp, const void *X, int64_t ldx,
                    const void *Y, int64_t ldy) {
  if (plan->d != 4096) return false;
  if (plan->algo == HARP_ALGO_GENERIC) return false;
  if (hp.npass != 3) return false;
  for (int p = 0; p < 3; ++p)
    if (hp.pass[p].kind != (p == 2 ? PASS_POW2_LIFT_LD : PASS_POW2_LIFT) || hp.pass[p].k != 4)
      return false;
  // pass strides must be the ones the kernel is compiled for (1, 16, 256 or reversed)
  const bool trn = hp.pass[0].desc != 0;
  for (int p = 0; p < 3; ++p)
    if (hp.pass[p].S != (1 << (4 * (trn ? 2 - p : p)))) return false;
  if ((ldx % 8) || (ldy % 8) || ((uintptr_t)X % 16) || ((uintptr_t)Y % 16)) return false;
  return true;
}

harp_status_t launch_pipe_kernel(const harp_plan *plan, const HostProgram &hp, const void *X,
                                 int64_t ldx, void *Y, int64_t ldy, int64_t n, int R,
                                 hipStream_t stream) {
  (void)plan;
  const bool trn = hp.prog.pass[0].desc != 0;
  if (trn) return launch_pipe_inst<4, 4, 4, true>(hp.dev, X, ldx, Y, ldy, n, R, stream);
  return launch_pipe_inst<4, 4, 4, false>(hp.dev, X, ldx, Y, ldy, n, R, stream);
}

}  // namespace harp
