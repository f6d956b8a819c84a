// Row-pipelined kernel for radix-2 chains of orthogonal blocks on rows, or contiguous row
// chunks, of 2^(K0+K1+K2) = 2048 or 4096 coordinates; bf16 or float32 on either side.  Every
// stage but the last is executed as two shears with deferred output scales (or, as the plan
// builder's fallback, three lifting steps), the last as a dense 2x2 that also carries all
// pending scales and signs, so the inner loop is fused multiply-adds only.  The second kernel of this file covers chunks of 256 / 512 / 1024 coordinates with one
// wave per window (see harp_wave_kernel below).
//
// The 10..12 stages are cut into three passes of K0, K1, K2 consecutive stages.  A workgroup
// has three wave groups of d/16 threads; group g executes pass g and nothing else, so a thread
// keeps the rotation parameters of its own 16 coordinates x K stages in registers for the
// whole launch (they are read from device memory exactly once per workgroup), and rows flow
// through the groups like an assembly line:
//
//    step k:  group 0  takes rows 2k, 2k+1 (prefetched from device memory one pair
//                      ahead), applies pass 0, writes them to LDS buffer A[k & 1]
//             group 1  reads pair k-1 from A[(k-1) & 1], applies pass 1, writes B[k & 1]
//             group 2  reads pair k-2 from B[(k-1) & 1], applies pass 2, rounds to the output
//                      type and stores the rows to device memory
//             one workgroup barrier
//
// so loads, the three passes and stores of different rows overlap, and the three groups give
// every SIMD three independent instruction streams.  The stride permutations of Eq. (7)
// appear only as the LDS addresses a group reads and writes (Lemma 1 indexing); the LDS
// positions are swizzled so that the contiguous 16-float accesses of the stride-1 pass and
// the stride-16 / stride-256 accesses of the other passes are all free of bank conflicts.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "harp_internal.h"

namespace harp {

namespace {

// parameter images live in device (global) memory: say so, so that the loads are global loads
// with a scalar base rather than generic-address loads
typedef const __attribute__((address_space(1))) float *gparams_t;

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
// per pair follow the (K-1) * P lifted values.  With SC a stage is two shears with deferred
// output scales instead: (x0, x1) <- (x0 + a x1, x1 + b x0), same parameter positions.
template <int K, bool DESC, bool LD, bool SC>
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
          if (SC) {
            x[j0] = fmaf(a, x1, x0);
            x[j1] = fmaf(b, x0, x1);
          } else {
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
}

// Element I/O of the first and last group.  NRAW = dwords a thread keeps per prefetched row.
template <typename T, bool CONTIG>
struct RowIo;

template <>
struct RowIo<uint16_t, true> {      // 16 contiguous bf16 (or 2 x 8): two 16-byte accesses
  static constexpr int NRAW = 8;
  template <class OFF>
  __device__ static __forceinline__ void load(const uint16_t *xr, OFF off, uint32_t (&raw)[NRAW]) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint4 v = *reinterpret_cast<const uint4 *>(xr + off(8 * h));
      raw[4 * h + 0] = v.x; raw[4 * h + 1] = v.y; raw[4 * h + 2] = v.z; raw[4 * h + 3] = v.w;
    }
  }
  __device__ static __forceinline__ void unpack(const uint32_t (&raw)[NRAW], float (&x)[16]) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      x[2 * m] = __uint_as_float(raw[m] << 16);
      x[2 * m + 1] = __uint_as_float(raw[m] & 0xffff0000u);
    }
  }
  template <class OFF>
  __device__ static __forceinline__ void store(uint16_t *yr, OFF off, const float (&x)[16]) {
    uint32_t w[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) w[m] = cvt_pk_bf16(x[2 * m], x[2 * m + 1]);
#pragma unroll
    for (int h = 0; h < 2; ++h)
      *reinterpret_cast<uint4 *>(yr + off(8 * h)) =
          make_uint4(w[4 * h], w[4 * h + 1], w[4 * h + 2], w[4 * h + 3]);
  }
  // the same with the sign bits of the packed elements flipped where flip[m] has them set
  template <class OFF>
  __device__ static __forceinline__ void store_flipped(uint16_t *yr, OFF off, const float (&x)[16],
                                                       const uint32_t (&flip)[8]) {
    uint32_t w[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) w[m] = cvt_pk_bf16(x[2 * m], x[2 * m + 1]) ^ flip[m];
#pragma unroll
    for (int h = 0; h < 2; ++h)
      *reinterpret_cast<uint4 *>(yr + off(8 * h)) =
          make_uint4(w[4 * h], w[4 * h + 1], w[4 * h + 2], w[4 * h + 3]);
  }
};

// 16 contiguous block-scaled halves = one aligned segment: two 16-byte accesses and the
// segment's exponent byte, which lies d halves behind the start of the row (xr = row start)
template <>
struct RowIo<zh16, true> {
  static constexpr int NRAW = 9;
  template <class OFF>
  __device__ static __forceinline__ void load_z(const zh16 *xr, OFF off, int d, uint32_t (&raw)[NRAW]) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint4 v = *reinterpret_cast<const uint4 *>(xr + off(8 * h));
      raw[4 * h + 0] = v.x; raw[4 * h + 1] = v.y; raw[4 * h + 2] = v.z; raw[4 * h + 3] = v.w;
    }
    raw[8] = reinterpret_cast<const uint8_t *>(xr + d)[off(0) >> 4];
  }
  __device__ static __forceinline__ void unpack(const uint32_t (&raw)[NRAW], float (&x)[16]) {
    const float sc = z16_up(raw[8]);
#pragma unroll
    for (int m = 0; m < 8; ++m) z16_unpack(raw[m], sc, x[2 * m], x[2 * m + 1]);
  }
  template <class OFF>
  __device__ static __forceinline__ void store_z(zh16 *yr, OFF off, int d, const float (&x)[16]) {
    float mx = fabsf(x[0]);
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(mx, fabsf(x[e]));
    const uint32_t ex = z16_exponent(mx);
    const float f = z16_down(ex);
    uint32_t w[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) w[m] = z16_pack(x[2 * m] * f, x[2 * m + 1] * f);
#pragma unroll
    for (int h = 0; h < 2; ++h)
      *reinterpret_cast<uint4 *>(yr + off(8 * h)) =
          make_uint4(w[4 * h], w[4 * h + 1], w[4 * h + 2], w[4 * h + 3]);
    reinterpret_cast<uint8_t *>(yr + d)[off(0) >> 4] = (uint8_t)ex;
  }
};

template <>
struct RowIo<uint16_t, false> {     // 16 single bf16 at the pass stride
  static constexpr int NRAW = 16;
  template <class OFF>
  __device__ static __forceinline__ void load(const uint16_t *xr, OFF off, uint32_t (&raw)[NRAW]) {
#pragma unroll
    for (int e = 0; e < 16; ++e) raw[e] = xr[off(e)];
  }
  __device__ static __forceinline__ void unpack(const uint32_t (&raw)[NRAW], float (&x)[16]) {
#pragma unroll
    for (int e = 0; e < 16; ++e) x[e] = __uint_as_float(raw[e] << 16);
  }
  template <class OFF>
  __device__ static __forceinline__ void store(uint16_t *yr, OFF off, const float (&x)[16]) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const uint32_t w = cvt_pk_bf16(x[2 * m], x[2 * m + 1]);
      yr[off(2 * m)] = (uint16_t)(w & 0xffffu);
      yr[off(2 * m + 1)] = (uint16_t)(w >> 16);
    }
  }
};

template <>
struct RowIo<float, true> {         // 16 contiguous floats (or 2 x 8): four 16-byte accesses
  static constexpr int NRAW = 16;
  template <class OFF>
  __device__ static __forceinline__ void load(const float *xr, OFF off, uint32_t (&raw)[NRAW]) {
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const uint4 v = *reinterpret_cast<const uint4 *>(xr + off(4 * h));
      raw[4 * h + 0] = v.x; raw[4 * h + 1] = v.y; raw[4 * h + 2] = v.z; raw[4 * h + 3] = v.w;
    }
  }
  __device__ static __forceinline__ void unpack(const uint32_t (&raw)[NRAW], float (&x)[16]) {
#pragma unroll
    for (int e = 0; e < 16; ++e) x[e] = __uint_as_float(raw[e]);
  }
  template <class OFF>
  __device__ static __forceinline__ void store(float *yr, OFF off, const float (&x)[16]) {
#pragma unroll
    for (int h = 0; h < 4; ++h)
      *reinterpret_cast<float4 *>(yr + off(4 * h)) =
          make_float4(x[4 * h], x[4 * h + 1], x[4 * h + 2], x[4 * h + 3]);
  }
};

template <>
struct RowIo<float, false> {        // 16 single floats at the pass stride
  static constexpr int NRAW = 16;
  template <class OFF>
  __device__ static __forceinline__ void load(const float *xr, OFF off, uint32_t (&raw)[NRAW]) {
#pragma unroll
    for (int e = 0; e < 16; ++e) raw[e] = __float_as_uint(xr[off(e)]);
  }
  __device__ static __forceinline__ void unpack(const uint32_t (&raw)[NRAW], float (&x)[16]) {
#pragma unroll
    for (int e = 0; e < 16; ++e) x[e] = __uint_as_float(raw[e]);
  }
  template <class OFF>
  __device__ static __forceinline__ void store(float *yr, OFF off, const float (&x)[16]) {
#pragma unroll
    for (int e = 0; e < 16; ++e) yr[off(e)] = x[e];
  }
};

// Body of one wave group.  ROLE 0 = first pass (reads device memory), 1 = middle, 2 = last
// (writes device memory; with LD its K-th stage is the program's last and is dense).  LOGS =
// log2 of the stride of the pass's lowest digit; the pass with LOGS == 0 touches contiguous
// coordinates (16-byte vector accesses), the others touch single coordinates.  kch = index of
// the chunk of D coordinates this workgroup works on (0 when D is the whole row).
// A step moves a PAIR of rows through every group: group g works on pair k - g at step k, one
// barrier per step, npairs + 2 steps for every group.  Inside a wave the LDS reads of the
// second row and the LDS writes of the first overlap with arithmetic.  Buffers hold two rows
// per parity: row r of the pair at + r * ROWBUF.
template <typename TI, typename TO, int K, int LOGS, bool DESC, int ROLE, bool LD, bool SC, int D>
__device__ __forceinline__ void pipe_group(const PassDesc &pd, const int t, const int kch,
                                            const float *rd_buf, float *wr_buf,
                                            const TI *__restrict__ X, const int64_t ldx,
                                            TO *__restrict__ Y, const int64_t ldy, const int nr) {
  constexpr int P = 1 << K, SPT = 16 / P, TG = D / 16, NV = (K + (LD ? 1 : 0)) * P;
  constexpr int ROWBUF = (D / 256) * 272;
  constexpr int S = 1 << LOGS;
  constexpr bool CONTIG = (LOGS == 0);
  using In = RowIo<TI, CONTIG>;
  using Out = RowIo<TO, CONTIG>;
  constexpr int NRAW = In::NRAW;
  // One pair of rows is prefetched ahead.  Two pairs measured 0.7 us slower at 8 rows per tile
  // (the first pair then queues behind twice the data at launch) and no faster at 64.
  constexpr int PFP = 1;
  const unsigned nq = (unsigned)pd.nq;
  const unsigned qoff = (unsigned)kch * (D / P);
  const float *__restrict__ params = pd.params;

  unsigned base[SPT];
#pragma unroll
  for (int u = 0; u < SPT; ++u) {
    const unsigned q = (unsigned)t + u * TG;
    const unsigned hi = q >> LOGS, lo = q & (S - 1);
    base[u] = ((hi << K) << LOGS) | lo;
  }
  auto lds_off = [&](int e) -> int {
    const int u = e / P, j = e % P;
    return phys_index((int)(base[u] | ((unsigned)j << LOGS)));
  };
  auto glb_off = [&](int e) -> unsigned {
    const int u = e / P, j = e % P;
    return base[u] | ((unsigned)j << LOGS);
  };

  // first rows before the parameters: their device-memory latency is the longer one
  uint32_t pre[2 * PFP][NRAW];
  if (ROLE == 0) {
#pragma unroll
    for (int s = 0; s < 2 * PFP; ++s) {
#pragma unroll
      for (int m = 0; m < NRAW; ++m) pre[s][m] = 0u;
      if (s < nr) In::load(X + (int64_t)s * ldx, glb_off, pre[s]);
    }
  }
  float prm[SPT * NV];
#pragma unroll
  for (int u = 0; u < SPT; ++u) {
    const unsigned q = (unsigned)t + u * TG;
#pragma unroll
    for (int v = 0; v < NV; ++v) prm[u * NV + v] = params[(unsigned)v * nq + qoff + q];
  }

  auto lds_read = [&](const float *b, float (&x)[16]) {
    if (CONTIG) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float4 f = *reinterpret_cast<const float4 *>(b + lds_off(4 * c));
        x[4 * c] = f.x; x[4 * c + 1] = f.y; x[4 * c + 2] = f.z; x[4 * c + 3] = f.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) x[e] = b[lds_off(e)];
    }
  };
  auto lds_write = [&](float *b, const float (&x)[16]) {
    if (CONTIG) {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        *reinterpret_cast<float4 *>(b + lds_off(4 * c)) =
            make_float4(x[4 * c], x[4 * c + 1], x[4 * c + 2], x[4 * c + 3]);
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) b[lds_off(e)] = x[e];
    }
  };

  // Last group, float32 output, contiguous pass: a thread's 16-byte stores would sit 64 bytes
  // apart from its neighbours' (the one slow store pattern measured on this chip, about 60 % of
  // the rate of any other; bf16 rows, 32 bytes apart, measured 7 % slower with the detour than
  // without, and the same detour on the float32 LOADS of a contiguous first pass gained
  // nothing), so the row goes once more through LDS -- through the
  // positions this wave has just read its input from, which nobody else touches before the
  // next barrier -- and leaves with 1 KB of consecutive addresses per store instruction.
  constexpr bool kRelayout = (ROLE == 2) && CONTIG && (sizeof(TO) == 4);
  auto store_relayout = [&](float *region, const float (&x)[16], TO *yrow) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      *reinterpret_cast<float4 *>(region + lds_off(4 * c)) =
          make_float4(x[4 * c], x[4 * c + 1], x[4 * c + 2], x[4 * c + 3]);
    // the region is private to this wave and LDS serves a wave's accesses in order
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const unsigned lane = (unsigned)t & 63u, w0 = (unsigned)t & ~63u;
#pragma unroll
    for (int u = 0; u < SPT; ++u) {
      const unsigned run = (w0 + (unsigned)u * TG) * P;     // 64 * P consecutive coordinates
#pragma unroll
      for (int g = 0; g < P / 4; ++g) {
        const unsigned coord = run + (unsigned)g * 256u + 4u * lane;
        const float4 f = *reinterpret_cast<const float4 *>(region + phys_index((int)coord));
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(yrow) + coord) = f;
      }
    }
    asm volatile("" ::: "memory");
  };

  const int npairs = (nr + 1) >> 1;
  const int nsteps = npairs + 2;   // group g works on pair k - g at step k; one barrier per step
  for (int k0 = 0; k0 < nsteps; k0 += 2) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int k = k0 + s;
      if (k >= nsteps) break;
      const int pr = k - ROLE;
      if (pr >= 0 && pr < npairs) {
        const int r0 = 2 * pr;
        const bool two = r0 + 1 < nr;
        float xa[16], xb[16];
        if (ROLE == 0) {
          const int slot = (PFP == 2) ? 2 * s : 0;   // pair index parity == step parity here
          In::unpack(pre[slot], xa);
          In::unpack(pre[slot + 1], xb);
          const int rn = r0 + 2 * PFP;
          if (rn < nr) In::load(X + (int64_t)rn * ldx, glb_off, pre[slot]);
          if (rn + 1 < nr) In::load(X + (int64_t)(rn + 1) * ldx, glb_off, pre[slot + 1]);
        } else {
          const float *b = rd_buf + ((s + 1) & 1) * (2 * ROWBUF);   // written in step k - 1
          lds_read(b, xa);
          lds_read(b + ROWBUF, xb);
        }
        float *wb = (ROLE == 2) ? nullptr : wr_buf + (s & 1) * (2 * ROWBUF);
        // input half of this step (groups 1, 2); reused as staging by the re-laid-out store
        float *stage = (ROLE == 0) ? nullptr
                                   : const_cast<float *>(rd_buf) + ((s + 1) & 1) * (2 * ROWBUF);
        lift_stages<K, DESC, LD, SC>(xa, prm);
        if (ROLE == 2) {
          if (kRelayout) store_relayout(stage, xa, Y + (int64_t)r0 * ldy);
          else Out::store(Y + (int64_t)r0 * ldy, glb_off, xa);
        } else {
          lds_write(wb, xa);
        }
        lift_stages<K, DESC, LD, SC>(xb, prm);
        if (ROLE == 2) {
          if (two) {
            if (kRelayout) store_relayout(stage + ROWBUF, xb, Y + (int64_t)(r0 + 1) * ldy);
            else Out::store(Y + (int64_t)(r0 + 1) * ldy, glb_off, xb);
          }
        } else {
          lds_write(wb + ROWBUF, xb);
        }
      }
      __syncthreads();
    }
  }
}

// Workgroup -> (chunk kch, tile of R rows).  nchunk = chunks per row (1: D is the whole row).
// The three chunk-local passes are prog.pass[p0 .. p0+2].
template <typename TI, typename TO, int K0, int K1, int K2, bool TRN, bool LD, bool SC>
__global__ __launch_bounds__(3 << (K0 + K1 + K2 - 4)) void harp_pipe_kernel(
    const TI *__restrict__ X, int64_t ldx, TO *__restrict__ Y, int64_t ldy, int64_t n, int R,
    int nchunk, const Program *__restrict__ progp, int p0) {
  constexpr int D = 1 << (K0 + K1 + K2), TG = D / 16, ROWBUF = (D / 256) * 272;
  __shared__ float bufA[4 * ROWBUF];
  __shared__ float bufB[4 * ROWBUF];
  const int g = __builtin_amdgcn_readfirstlane((int)threadIdx.x / TG);  // wave-uniform
  const int t = (int)threadIdx.x % TG;
  const int kch = (int)(blockIdx.x % (unsigned)nchunk);
  const int64_t row0 = (int64_t)(blockIdx.x / (unsigned)nchunk) * R;
  const int nr = (int)((n - row0 < R) ? (n - row0) : R);
  const Program &prog = *progp;
  const TI *Xt = X + row0 * ldx + (int64_t)kch * D;
  TO *Yt = Y + row0 * ldy + (int64_t)kch * D;
  // stride of each pass's lowest digit: ascending for apply, descending for apply_transpose
  constexpr int LS0 = TRN ? K1 + K2 : 0, LS1 = TRN ? K2 : K0, LS2 = TRN ? 0 : K0 + K1;
  if (g == 0)
    pipe_group<TI, TO, K0, LS0, TRN, 0, false, SC, D>(prog.pass[p0], t, kch, nullptr, bufA, Xt,
                                                       ldx, Yt, ldy, nr);
  else if (g == 1)
    pipe_group<TI, TO, K1, LS1, TRN, 1, false, SC, D>(prog.pass[p0 + 1], t, kch, bufA, bufB, Xt,
                                                       ldx, Yt, ldy, nr);
  else
    pipe_group<TI, TO, K2, LS2, TRN, 2, LD, SC, D>(prog.pass[p0 + 2], t, kch, bufB, nullptr, Xt,
                                                    ldx, Yt, ldy, nr);
}

// ------------------------------------------------------------------------------------------
// Wave-local kernel for radix-2 chains on chunks of 256 / 512 / 1024 coordinates.
//
// One wave (a workgroup of 64 threads) owns a window of 1024 consecutive coordinates of the row
// -- 4, 2 or 1 whole chunks -- and walks down R rows.  A thread keeps the parameters of ALL
// passes of its 16 coordinates in registers (128..176 values), so they are read once per
// workgroup; a row is loaded with 16-byte accesses (next row prefetched), goes through the 2 or
// 3 passes with an LDS exchange between them (private to the wave: no other wave waits), and
// is stored with 16-byte accesses (when the last pass is a strided one, the last exchange puts
// the row into a layout in which every store instruction writes 1 KB of consecutive addresses).  Used for the 2^8 part of d = 11008 = 2^8 * 43 and for
// short rows.
template <int K, int LOGS, bool LD>
struct WavePass {
  static constexpr int P = 1 << K, SPT = 16 / P, NV = (K + (LD ? 1 : 0)) * P, S = 1 << LOGS;
  float prm[SPT * NV];
  unsigned base[SPT];
  // window kg of the row; sub-tensors kg * (1024 / P) + t + 64 u of the row's pd.nq
  __device__ __forceinline__ void init(const PassDesc &pd, int t, int kg, bool with_params) {
    const unsigned nq = (unsigned)pd.nq, nqp = (unsigned)pd.nqp;
#pragma unroll
    for (int u = 0; u < SPT; ++u) {
      const unsigned ql = (unsigned)t + 64u * u;
      const unsigned qg = (unsigned)kg * (1024 / P) + ql;
      const bool ok = with_params && qg < nq;
      // tied parameters (Kronecker plans): every slice reads the one image, nqp a power of two
      const unsigned qp = pd.tied ? (qg & (nqp - 1u)) : qg;
#pragma unroll
      for (int v = 0; v < NV; ++v) prm[u * NV + v] = ok ? ((gparams_t)pd.params)[(unsigned)v * nqp + qp] : 0.0f;
      const unsigned hi = ql >> LOGS, lo = ql & (S - 1);
      base[u] = ((hi << K) << LOGS) | lo;
    }
  }
  __device__ __forceinline__ unsigned coord(int e) const {
    return base[e / P] | ((unsigned)(e % P) << LOGS);
  }
};

// Store layout of the wave kernel: a thread's 16 elements are 16-byte pieces (PIECE = 4 float32
// or 8 bf16 coordinates) placed so that one store instruction of the wave writes 1 KB of
// consecutive addresses: element e <-> coordinate (e / PIECE) * 64 * PIECE + PIECE * t + e % PIECE
// of the 1024-coordinate window.
template <typename TO>
struct WaveStoreLayout {
  static constexpr int PIECE = 16 / (int)sizeof(TO), NP = 16 / PIECE;
  static constexpr int S = 1, P = PIECE;   // contiguous groups of >= 4: 16-byte LDS reads
  unsigned t;
  __device__ __forceinline__ unsigned coord(int e) const {
    return (unsigned)(e / PIECE) * (64u * PIECE) + (unsigned)PIECE * t + (unsigned)(e % PIECE);
  }
  // pieces whose coordinates lie inside the row (valid = coordinates of the window inside it)
  __device__ __forceinline__ void store(TO *yw, const float (&x)[16], int valid) const;
  // block-scaled halves (yrow = start of the row, w0 = first coordinate of the window): a piece
  // is half a segment, the other half belongs to the neighbouring lane
  __device__ __forceinline__ void store_z16(zh16 *yrow, unsigned w0, int d, const float (&x)[16],
                                            int valid) const {
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      float mx = fabsf(x[8 * g]);
#pragma unroll
      for (int e = 1; e < 8; ++e) mx = fmaxf(mx, fabsf(x[8 * g + e]));
      const float other = __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(
          0, (int)__float_as_uint(mx), 0xB1 /* quad_perm [1,0,3,2] */, 0xf, 0xf, false));
      const uint32_t ex = z16_exponent(fmaxf(mx, other));
      const float f = z16_down(ex);
      const unsigned c = (unsigned)g * 512u + 8u * t;
      if ((int)c < valid) {
        *reinterpret_cast<uint4 *>(yrow + w0 + c) =
            make_uint4(z16_pack(x[8 * g] * f, x[8 * g + 1] * f), z16_pack(x[8 * g + 2] * f, x[8 * g + 3] * f),
                       z16_pack(x[8 * g + 4] * f, x[8 * g + 5] * f), z16_pack(x[8 * g + 6] * f, x[8 * g + 7] * f));
        if (!(t & 1u)) reinterpret_cast<uint8_t *>(yrow + d)[(w0 + c) >> 4] = (uint8_t)ex;
      }
    }
  }
  // bf16 only: sign bits of the packed elements flipped where flip[m] has them set
  __device__ __forceinline__ void store_flipped(uint16_t *yw, const float (&x)[16], int valid,
                                                const uint32_t (&flip)[8]) const {
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const unsigned c = coord(8 * g);
      if ((int)c < valid)
        *reinterpret_cast<uint4 *>(yw + c) =
            make_uint4(cvt_pk_bf16(x[8 * g], x[8 * g + 1]) ^ flip[4 * g],
                       cvt_pk_bf16(x[8 * g + 2], x[8 * g + 3]) ^ flip[4 * g + 1],
                       cvt_pk_bf16(x[8 * g + 4], x[8 * g + 5]) ^ flip[4 * g + 2],
                       cvt_pk_bf16(x[8 * g + 6], x[8 * g + 7]) ^ flip[4 * g + 3]);
    }
  }
};
template <>
__device__ __forceinline__ void WaveStoreLayout<float>::store(float *yw, const float (&x)[16],
                                                              int valid) const {
#pragma unroll
  for (int g = 0; g < NP; ++g) {
    const unsigned c = coord(PIECE * g);
    if ((int)c < valid)
      *reinterpret_cast<float4 *>(yw + c) =
          make_float4(x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]);
  }
}
template <>
__device__ __forceinline__ void WaveStoreLayout<uint16_t>::store(uint16_t *yw,
                                                                 const float (&x)[16],
                                                                 int valid) const {
#pragma unroll
  for (int g = 0; g < NP; ++g) {
    const unsigned c = coord(PIECE * g);
    if ((int)c < valid)
      *reinterpret_cast<uint4 *>(yw + c) =
          make_uint4(cvt_pk_bf16(x[8 * g], x[8 * g + 1]), cvt_pk_bf16(x[8 * g + 2], x[8 * g + 3]),
                     cvt_pk_bf16(x[8 * g + 4], x[8 * g + 5]), cvt_pk_bf16(x[8 * g + 6], x[8 * g + 7]));
  }
}

// x leaves layout A and comes back in layout B through the wave's LDS buffer
template <class PA, class PB>
__device__ __forceinline__ void wave_exchange(float (&x)[16], float *buf, const PA &a, const PB &b) {
  if (PA::S == 1 && PA::P >= 4) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      *reinterpret_cast<float4 *>(buf + phys_index((int)a.coord(4 * c))) =
          make_float4(x[4 * c], x[4 * c + 1], x[4 * c + 2], x[4 * c + 3]);
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e) buf[phys_index((int)a.coord(e))] = x[e];
  }
  __syncthreads();
  if (PB::S == 1 && PB::P >= 4) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float4 f = *reinterpret_cast<const float4 *>(buf + phys_index((int)b.coord(4 * c)));
      x[4 * c] = f.x; x[4 * c + 1] = f.y; x[4 * c + 2] = f.z; x[4 * c + 3] = f.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e) x[e] = buf[phys_index((int)b.coord(e))];
  }
  __syncthreads();
}

// SGN: the +-1 signs of the processor applied here instead of being folded into the stage
// parameters (plans with tied parameters): 1 = on the coordinates as loaded, 2 = as stored.
template <typename TI, typename TO, int K0, int K1, int K2, bool TRN, bool LD, bool SC, int SGN = 0>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void harp_wave_kernel(const TI *__restrict__ X, int64_t ldx,
                                                       TO *__restrict__ Y, int64_t ldy, int64_t n,
                                                       int R, int ngroups, int d,
                                                       const Program *__restrict__ progp, int p0,
                                                       const int8_t *__restrict__ signs = nullptr) {
  constexpr bool THREE = (K2 != 0);
  constexpr int LS0 = TRN ? K1 + K2 : 0, LS1 = TRN ? K2 : K0, LS2 = TRN ? 0 : K0 + K1;
  __shared__ float buf[(1024 / 256) * 272];
  const int t = threadIdx.x;
  const int kg = (int)(blockIdx.x % (unsigned)ngroups);
  const int64_t row0 = (int64_t)(blockIdx.x / (unsigned)ngroups) * R;
  const int nr = (int)((n - row0 < R) ? (n - row0) : R);
  const int w0 = kg * 1024;
  const int valid = (d - w0 < 1024) ? d - w0 : 1024;   // coordinates of the window inside the row
  const Program &prog = *progp;

  WavePass<K0, LS0, (!THREE && false)> pa;                // first pass is never the dense-ended one
  WavePass<K1, LS1, (!THREE && LD)> pb;
  WavePass<(THREE ? K2 : 1), (THREE ? LS2 : 0), (THREE && LD)> pc;
  WavePass<4, 0, false> io;                               // 16 contiguous coordinates per thread
  pa.init(prog.pass[p0], t, kg, true);
  pb.init(prog.pass[p0 + 1], t, kg, true);
  if (THREE) pc.init(prog.pass[p0 + 2], t, kg, true);
  io.init(prog.pass[p0], t, kg, false);
  WaveStoreLayout<TO> sl{(unsigned)t};
  // the last pass leaves the row in the load layout only when it is the (4 stages, stride 1) one
  constexpr bool kLastIsIo = THREE ? (K2 == 4 && LS2 == 0) : (K1 == 4 && LS1 == 0);
  const bool active = 16 * t < valid;
  auto goff = [&](int e) -> unsigned { return (unsigned)w0 + io.coord(e); };
  // Signs of the thread's 16 coordinates in the layout they are applied in.  bf16 side: as
  // flip words for the packed pairs (bit 15 = element 2m, bit 31 = element 2m + 1), one
  // exclusive-or per two coordinates; float32 side: one bit per element in a single register
  // (sixteen flip words would push the three-pass instances past 256 registers).
  constexpr bool kFlipIn = (SGN == 1), kFlipOut = (SGN == 2);
  constexpr bool kPackedFlip = (kFlipIn && sizeof(TI) == 2) || (kFlipOut && sizeof(TO) == 2);
  uint32_t sgw[kPackedFlip ? 8 : 1] = {};
  uint32_t sgm = 0;
  if (SGN) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const unsigned c = (kFlipIn || kLastIsIo) ? io.coord(e) : sl.coord(e);
      const uint32_t neg = ((int)c < valid && signs[(unsigned)w0 + c] < 0) ? 1u : 0u;
      if (kPackedFlip) sgw[kPackedFlip ? e / 2 : 0] |= neg << (15 + 16 * (e & 1));
      else sgm |= neg << e;
    }
  }
  auto flip_f32 = [&](float (&x)[16]) {   // sign from (x ^ shifted mask), magnitude from x
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const uint32_t u = __float_as_uint(x[e]);
      x[e] = __uint_as_float((u & 0x7fffffffu) | ((u ^ (sgm << (31 - e))) & 0x80000000u));
    }
  };
  using In = RowIo<TI, true>;
  using Out = RowIo<TO, true>;
  constexpr int NRAW = In::NRAW;
  constexpr bool kZIn = std::is_same<TI, zh16>::value, kZOut = std::is_same<TO, zh16>::value;
  // Rows requested ahead: two, but one when the input is float32 and there are three passes.
  // That combination (the transposed chunk kernels of split programs) otherwise needs 264 to
  // 277 registers per thread, past the 256 at which a second wave still fits on a SIMD, and ran
  // 30-45 % slower than its forward counterpart for that reason alone.
  constexpr int PF = (sizeof(TI) == 4 && THREE) ? 1 : 2;
  uint32_t pre[PF][NRAW];
#pragma unroll
  for (int s = 0; s < PF; ++s) {
#pragma unroll
    for (int m = 0; m < NRAW; ++m) pre[s][m] = 0u;
    if (active && s < nr) {
      if constexpr (kZIn) In::load_z(X + (row0 + s) * ldx, goff, d, pre[s]);
      else In::load(X + (row0 + s) * ldx, goff, pre[s]);
    }
  }

  for (int r0 = 0; r0 < nr; r0 += PF) {
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      const int r = r0 + s;
      if (r >= nr) break;
      float x[16];
      if constexpr (kFlipIn && kPackedFlip) {
        uint32_t w[NRAW];
#pragma unroll
        for (int m = 0; m < NRAW; ++m) w[m] = pre[s][m] ^ sgw[m & 7];
        In::unpack(w, x);
      } else {
        In::unpack(pre[s], x);
      }
      if (active && r + PF < nr) {
        if constexpr (kZIn) In::load_z(X + (row0 + r + PF) * ldx, goff, d, pre[s]);
        else In::load(X + (row0 + r + PF) * ldx, goff, pre[s]);
      }
      if (kFlipIn && !kPackedFlip) flip_f32(x);

      if (!(K0 == 4 && LS0 == 0)) wave_exchange(x, buf, io, pa);
      lift_stages<K0, TRN, false, SC>(x, pa.prm);
      wave_exchange(x, buf, pa, pb);
      lift_stages<K1, TRN, (!THREE && LD), SC>(x, pb.prm);
      if (THREE) {
        wave_exchange(x, buf, pb, pc);
        lift_stages<(THREE ? K2 : 1), TRN, (THREE && LD), SC>(x, pc.prm);
        if (!kLastIsIo) wave_exchange(x, buf, pc, sl);
      } else {
        if (!kLastIsIo) wave_exchange(x, buf, pb, sl);
      }
      if (kFlipOut && !kPackedFlip) flip_f32(x);
      if constexpr (kFlipOut && kPackedFlip) {
        if (kLastIsIo) {
          if (active) Out::store_flipped(Y + (row0 + r) * ldy, goff, x, sgw);
        } else {
          sl.store_flipped(Y + (row0 + r) * ldy + w0, x, valid, sgw);
        }
      } else if constexpr (kZOut) {
        if (kLastIsIo) {
          if (active) Out::store_z(Y + (row0 + r) * ldy, goff, d, x);
        } else {
          sl.store_z16(Y + (row0 + r) * ldy, (unsigned)w0, d, x, valid);
        }
      } else if (kLastIsIo) {
        if (active) Out::store(Y + (row0 + r) * ldy, goff, x);
      } else {
        sl.store(Y + (row0 + r) * ldy + w0, x, valid);
      }
    }
  }
}

// Passes ps[0 .. np): all lifted, or all in the two-shear form; only the last may end with the
// program's dense stage.
bool pow2_family(const PassDesc *ps, int np, bool *ld, bool *sc) {
  const int last = ps[np - 1].kind;
  *sc = (last == PASS_POW2_SCALED || last == PASS_POW2_SCALED_LD);
  const int plain = *sc ? PASS_POW2_SCALED : PASS_POW2_LIFT;
  const int ended = *sc ? PASS_POW2_SCALED_LD : PASS_POW2_LIFT_LD;
  for (int p = 0; p < np - 1; ++p)
    if (ps[p].kind != plain) return false;
  if (last != plain && last != ended) return false;
  *ld = (last == ended);
  return true;
}

struct WaveArgs {
  const Program *dprog;
  int p0;
  const void *X;
  int64_t ldx;
  void *Y;
  int64_t ldy;
  int64_t n;
  int R;
  int d;
  hipStream_t stream;
  const int8_t *signs;
};

template <typename TI, typename TO, int K0, int K1, int K2, bool TRN, bool LD, bool SC, int SGN = 0>
harp_status_t launch_wave_inst(const WaveArgs &a) {
  const int ngroups = (a.d + 1023) / 1024;
  const int64_t tiles = ((a.n + a.R - 1) / a.R) * ngroups;
  if (tiles > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((harp_wave_kernel<TI, TO, K0, K1, K2, TRN, LD, SC, SGN>), dim3((unsigned)tiles),
                     dim3(64), 0, a.stream, (const TI *)a.X, a.ldx, (TO *)a.Y, a.ldy, a.n, a.R,
                     ngroups, a.d, a.dprog, a.p0, a.signs);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

// Plans with tied parameters: two-shear form with a dense stage at the end of the slices in both
// directions; forward = the slices come first (signs on the loaded coordinates), transposed =
// the slices come last (signs on the stored coordinates).  sgn = false: the plan has no signs.
template <typename TI, typename TO, int K0, int K1, int K2, bool TRN>
harp_status_t launch_wave_tied(const WaveArgs &a, bool sgn) {
  return sgn ? launch_wave_inst<TI, TO, K0, K1, K2, TRN, true, true, (TRN ? 2 : 1)>(a)
             : launch_wave_inst<TI, TO, K0, K1, K2, TRN, true, true, 0>(a);
}

template <typename TI, typename TO>
harp_status_t launch_wave_tied_io(const WaveArgs &a, int logc, bool trn, bool sgn) {
  if (logc == 8)
    return trn ? launch_wave_tied<TI, TO, 4, 4, 0, true>(a, sgn) : launch_wave_tied<TI, TO, 4, 4, 0, false>(a, sgn);
  if (logc == 9)
    return trn ? launch_wave_tied<TI, TO, 3, 3, 3, true>(a, sgn) : launch_wave_tied<TI, TO, 3, 3, 3, false>(a, sgn);
  if (logc == 10)
    return trn ? launch_wave_tied<TI, TO, 3, 3, 4, true>(a, sgn) : launch_wave_tied<TI, TO, 4, 3, 3, false>(a, sgn);
  return HARP_ERR_UNSUPPORTED;
}

template <typename TI, typename TO, int K0, int K1, int K2, bool SC, bool TRN>
harp_status_t launch_wave_form(const WaveArgs &a, bool ld) {
  if (TRN)
    return ld ? launch_wave_inst<TI, TO, K0, K1, K2, TRN, true, SC>(a) : HARP_ERR_UNSUPPORTED;
  return ld ? launch_wave_inst<TI, TO, K0, K1, K2, TRN, true, SC>(a)
            : launch_wave_inst<TI, TO, K0, K1, K2, TRN, (TRN ? true : false), SC>(a);
}

template <typename TI, typename TO, int K0, int K1, int K2, bool TRN>
harp_status_t launch_wave_dir(const WaveArgs &a, bool ld, bool sc) {
  return sc ? launch_wave_form<TI, TO, K0, K1, K2, true, TRN>(a, ld)
            : launch_wave_form<TI, TO, K0, K1, K2, false, TRN>(a, ld);
}

template <typename TI, typename TO>
harp_status_t launch_wave_io(const WaveArgs &a, int logc, bool trn, bool ld, bool sc) {
  if (logc == 8)
    return trn ? launch_wave_dir<TI, TO, 4, 4, 0, true>(a, ld, sc)
               : launch_wave_dir<TI, TO, 4, 4, 0, false>(a, ld, sc);
  if (logc == 9)
    return trn ? launch_wave_dir<TI, TO, 3, 3, 3, true>(a, ld, sc)
               : launch_wave_dir<TI, TO, 3, 3, 3, false>(a, ld, sc);
  if (logc == 10)   // the pass on the four lowest digits comes first going up, last going down
    return trn ? launch_wave_dir<TI, TO, 3, 3, 4, true>(a, ld, sc)
               : launch_wave_dir<TI, TO, 4, 3, 3, false>(a, ld, sc);
  return HARP_ERR_UNSUPPORTED;
}

// Passes [p0, p0+np) must be the lifted radix-2 passes (4,4), (3,3,3) or (4,3,3) -- (3,3,4) in a
// transposed program -- of a chunk of 256 / 512 / 1024 coordinates with the strides the kernel
// is compiled for.
bool wave_decode(const Program &pg, int p0, int np, int chunk, int *logc, bool *trn, bool *ld,
                 bool *sc) {
  if (np != 2 && np != 3) return false;
  const PassDesc *ps = pg.pass + p0;
  const int k0 = ps[0].k, k1 = ps[1].k, k2 = (np == 3) ? ps[2].k : 0;
  const int lc = k0 + k1 + k2;
  const bool down = ps[0].desc != 0;
  if (!((lc == 8 && k0 == 4 && k1 == 4 && np == 2) || (lc == 9 && k0 == 3 && k1 == 3 && k2 == 3) ||
        (lc == 10 && !down && k0 == 4 && k1 == 3 && k2 == 3) ||
        (lc == 10 && down && k0 == 3 && k1 == 3 && k2 == 4)))
    return false;
  if (chunk != (1 << lc)) return false;
  if (!pow2_family(ps, np, ld, sc)) return false;
  *trn = down;
  for (int p = 1; p < np; ++p)
    if (ps[p].desc != ps[0].desc) return false;
  if (*trn && !*ld) return false;
  int below = 0;   // log2 stride expected for each pass
  for (int p = 0; p < np; ++p) {
    const int pe = *trn ? np - 1 - p : p;   // passes from the lowest digits upwards
    if (ps[pe].S != (1 << below)) return false;
    below += ps[pe].k;
  }
  *logc = lc;
  return true;
}

struct PipeArgs {
  const Program *dprog;
  int p0;
  const void *X;
  int64_t ldx;
  void *Y;
  int64_t ldy;
  int64_t n;
  int R;
  int nchunk;
  hipStream_t stream;
};

template <typename TI, typename TO, int K0, int K1, int K2, bool TRN, bool LD, bool SC>
harp_status_t launch_pipe_inst(const PipeArgs &a) {
  constexpr int NT = 3 << (K0 + K1 + K2 - 4);
  const int64_t tiles = ((a.n + a.R - 1) / a.R) * a.nchunk;
  if (tiles > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((harp_pipe_kernel<TI, TO, K0, K1, K2, TRN, LD, SC>), dim3((unsigned)tiles),
                     dim3(NT), 0, a.stream, (const TI *)a.X, a.ldx, (TO *)a.Y, a.ldy, a.n, a.R,
                     a.nchunk, a.dprog, a.p0);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

template <typename TI, typename TO, int K0, int K1, int K2, bool SC>
harp_status_t launch_pipe_form(const PipeArgs &a, bool trn, bool ld) {
  if (trn)
    return ld ? launch_pipe_inst<TI, TO, K0, K1, K2, true, true, SC>(a) : HARP_ERR_UNSUPPORTED;
  return ld ? launch_pipe_inst<TI, TO, K0, K1, K2, false, true, SC>(a)
            : launch_pipe_inst<TI, TO, K0, K1, K2, false, false, SC>(a);
}

template <typename TI, typename TO, int K0, int K1, int K2>
harp_status_t launch_pipe_dir(const PipeArgs &a, bool trn, bool ld, bool sc) {
  return sc ? launch_pipe_form<TI, TO, K0, K1, K2, true>(a, trn, ld)
            : launch_pipe_form<TI, TO, K0, K1, K2, false>(a, trn, ld);
}

template <typename TI, typename TO>
harp_status_t launch_pipe_io(const PipeArgs &a, int logd, bool trn, bool ld, bool sc) {
  if (logd == 12) return launch_pipe_dir<TI, TO, 4, 4, 4>(a, trn, ld, sc);
  if (logd == 11) return launch_pipe_dir<TI, TO, 4, 4, 3>(a, trn, ld, sc);
  return HARP_ERR_UNSUPPORTED;
}

// Decode the three passes [p0, p0+3): lifted radix-2 passes of (4,4,4) or (4,4,3) stages on a
// chunk of 2^12 / 2^11 coordinates with the strides the kernel is compiled for.
bool pipe_decode(const Program &pg, int p0, int np, int chunk, int *logd, bool *trn, bool *ld,
                 bool *sc) {
  if (np != 3) return false;
  const PassDesc *ps = pg.pass + p0;
  const int k0 = ps[0].k, k1 = ps[1].k, k2 = ps[2].k;
  if (!(k0 == 4 && k1 == 4 && (k2 == 4 || k2 == 3))) return false;
  if (chunk != (1 << (k0 + k1 + k2))) return false;
  if (!pow2_family(ps, 3, ld, sc)) return false;
  *trn = ps[0].desc != 0;
  if (ps[1].desc != ps[0].desc || ps[2].desc != ps[0].desc) return false;
  if (*trn && !*ld) return false;   // a transposed program always ends inside the chunk
  const int s0 = *trn ? (1 << (k1 + k2)) : 1, s1 = *trn ? (1 << k2) : (1 << k0);
  const int s2 = *trn ? 1 : (1 << (k0 + k1));
  if (ps[0].S != s0 || ps[1].S != s1 || ps[2].S != s2) return false;
  *logd = k0 + k1 + k2;
  return true;
}

}  // namespace

bool pipe_supported(const harp_plan *plan, const Program &pg, int p0, int np, int chunk,
                    const void *X, int64_t ldx, const void *Y, int64_t ldy) {
  if (plan->algo == HARP_ALGO_GENERIC) return false;
  int logd;
  bool trn, ld, sc;
  if (!pipe_decode(pg, p0, np, chunk, &logd, &trn, &ld, &sc)) return false;
  // 16-byte row accesses for either element type
  if ((ldx % 8) || (ldy % 8) || ((uintptr_t)X % 16) || ((uintptr_t)Y % 16)) return false;
  return true;
}

bool wave_supported(const harp_plan *plan, const Program &pg, int p0, int np, int chunk,
                    const void *X, int64_t ldx, const void *Y, int64_t ldy) {
  if (plan->algo == HARP_ALGO_GENERIC) return false;
  int logc;
  bool trn, ld, sc;
  if (!wave_decode(pg, p0, np, chunk, &logc, &trn, &ld, &sc)) return false;
  if ((ldx % 8) || (ldy % 8) || ((uintptr_t)X % 16) || ((uintptr_t)Y % 16)) return false;
  return true;
}

harp_status_t launch_wave_kernel(const harp_plan *plan, const HostProgram &hp, int p0, int np,
                                 int chunk, const void *X, int64_t ldx, harp_dtype_t dt_in,
                                 void *Y, int64_t ldy, harp_dtype_t dt_out, int64_t n,
                                 hipStream_t stream) {
  int logc;
  bool trn, ld, sc;
  if (!wave_decode(hp.prog, p0, np, chunk, &logc, &trn, &ld, &sc)) return HARP_ERR_UNSUPPORTED;
  const int64_t ngroups = (plan->d + 1023) / 1024;
  // about 6 waves per compute unit (a wave re-reads 36 KB of parameters: 16 rows per wave
  // measured 14 % faster than 8 at 2048 x 11008); 4 to 16 rows per wave
  int64_t R = plan->rows_override > 0 ? plan->rows_override
                                      : (n * ngroups + (int64_t)plan->num_cu * 6 - 1) /
                                            ((int64_t)plan->num_cu * 6);
  if (plan->rows_override <= 0 && R < 4) R = 4;
  if (plan->rows_override <= 0 && R > 16) R = 16;
  if (R > n) R = n;
  if (R < 1) R = 1;
  WaveArgs a{hp.dev, p0, X, ldx, Y, ldy, n, (int)R, (int)plan->d, stream, plan->dev_signs};
  if (plan->tied_K > 0) {
    // shear form with a dense stage at the end of the slices, in both directions
    if (!sc || !ld) return HARP_ERR_UNSUPPORTED;
    const bool sgn = plan->dev_signs != nullptr;
    if (dt_in == HARP_BF16 && dt_out == HARP_BF16) return launch_wave_tied_io<uint16_t, uint16_t>(a, logc, trn, sgn);
    if (dt_in == HARP_BF16 && dt_out == HARP_F32) return launch_wave_tied_io<uint16_t, float>(a, logc, trn, sgn);
    if (dt_in == HARP_F32 && dt_out == HARP_BF16) return launch_wave_tied_io<float, uint16_t>(a, logc, trn, sgn);
    return launch_wave_tied_io<float, float>(a, logc, trn, sgn);
  }
  // block-scaled half intermediate of a split program: written going up, read going down
  if ((int)dt_out == kDtZ16)
    return (dt_in == HARP_BF16 && !trn) ? launch_wave_io<uint16_t, zh16>(a, logc, false, ld, sc)
                                        : HARP_ERR_UNSUPPORTED;
  if ((int)dt_in == kDtZ16)
    return (dt_out == HARP_BF16 && trn) ? launch_wave_io<zh16, uint16_t>(a, logc, true, ld, sc)
                                        : HARP_ERR_UNSUPPORTED;
  if (dt_in == HARP_BF16 && dt_out == HARP_BF16)
    return launch_wave_io<uint16_t, uint16_t>(a, logc, trn, ld, sc);
  if (dt_in == HARP_BF16 && dt_out == HARP_F32)
    return launch_wave_io<uint16_t, float>(a, logc, trn, ld, sc);
  if (dt_in == HARP_F32 && dt_out == HARP_BF16)
    return launch_wave_io<float, uint16_t>(a, logc, trn, ld, sc);
  return launch_wave_io<float, float>(a, logc, trn, ld, sc);
}

harp_status_t launch_pipe_kernel(const harp_plan *plan, const HostProgram &hp, int p0, int chunk,
                                 const void *X, int64_t ldx, harp_dtype_t dt_in, void *Y,
                                 int64_t ldy, harp_dtype_t dt_out, int64_t n, int R,
                                 hipStream_t stream) {
  int logd;
  bool trn, ld, sc;
  if (!pipe_decode(hp.prog, p0, 3, chunk, &logd, &trn, &ld, &sc)) return HARP_ERR_UNSUPPORTED;
  PipeArgs a{hp.dev, p0, X, ldx, Y, ldy, n, R, (int)(plan->d / chunk), stream};
  if (dt_in == HARP_BF16 && dt_out == HARP_BF16)
    return launch_pipe_io<uint16_t, uint16_t>(a, logd, trn, ld, sc);
  if (dt_in == HARP_BF16 && dt_out == HARP_F32)
    return launch_pipe_io<uint16_t, float>(a, logd, trn, ld, sc);
  if (dt_in == HARP_F32 && dt_out == HARP_BF16)
    return launch_pipe_io<float, uint16_t>(a, logd, trn, ld, sc);
  return launch_pipe_io<float, float>(a, logd, trn, ld, sc);
}

}  // namespace harp
