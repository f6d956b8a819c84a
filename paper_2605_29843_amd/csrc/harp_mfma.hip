// Streamed pass of one large-radix stage (radix 9..64, e.g. the radix-43 stage of d = 11008)
// on the matrix cores.
//
// For every block c = q of the stage, the stage multiplies the row vector of the b coordinates
// base(q) + j*S by the dense b x b block (Alg. 1, blockwise multiplication): a batch of small
// GEMMs  Y[rows, b] = Z[rows, b] * K_q[b, b], one per q, with the rows of the batch as the M
// dimension -- a real dense contraction, 2*b flops per coordinate, which the vector ALUs cannot
// sustain at memory speed.  It runs on v_mfma_f32_16x16x16_bf16 with float32 accumulation.
// Operand narrowing (documented approximation): each float32 operand is split into two bf16
// terms, x = x_hi + x_lo, and x_hi*K_hi + x_lo*K_hi + x_hi*K_lo is accumulated (about 16
// significant bits per product).  The launcher only takes this form when the caller's element
// type is bf16.  With float32 on both sides of the call the same kernel runs on
// v_mfma_f32_16x16x4_f32 with unsplit float32 operands (F32 = true): a quarter of the k extent
// per instruction, still far below the time the rows take to stream.
//
// A workgroup of 16 waves owns 16 consecutive blocks q (same hi, consecutive lo: 64-byte
// contiguous runs in memory for every row and j) and walks down its rows 16 at a time:
//   global -> LDS tile[j][lo][row] (coalesced 16-byte loads, next chunk prefetched in registers)
//   wave w (block q0 + w): A = tile[:, w, :] split to bf16 hi/lo, B = its block, resident in
//   registers for the whole launch in MFMA lane layout (packed by the plan)
//   accumulators -> the same LDS tile positions (j' replaces j) -> coalesced stores.
//
// A workgroup touches only 64 (float32) or 32 (bf16) bytes of every 128-byte line it reads, so
// the 4 workgroups that share those lines (4 consecutive q tiles, same rows) are numbered to
// land on the same XCD next to each other in dispatch order (workgroup i runs on XCD i mod 8):
// the line is then fetched from device memory once and served to the other three from that
// XCD's L2.  Without this the kernel fetched 2.7 times its input (measured, FETCH_SIZE).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "harp_internal.h"

namespace harp {

namespace {

typedef short s4v __attribute__((ext_vector_type(4)));
typedef float f4v __attribute__((ext_vector_type(4)));

constexpr int kRC = 16;    // rows per chunk (the MFMA M dimension)
constexpr int kLS = 17;    // LDS stride between consecutive lo (16 rows + 1 pad)
constexpr int kJS = 276;   // LDS stride between consecutive j (16 * 17 + 4 pad; 4*kJS = 16 mod 32)

__device__ __forceinline__ uint32_t pk_bf16(float lo, float hi) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  bf2 v;
  v.x = (__bf16)lo;
  v.y = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

// x[0..3] -> bf16 hi part and bf16 lo part (x - hi), each as 4 packed bf16
__device__ __forceinline__ void split4(const float (&x)[4], s4v &hi, s4v &lo) {
  const uint32_t h0 = pk_bf16(x[0], x[1]), h1 = pk_bf16(x[2], x[3]);
  const float r0 = x[0] - __uint_as_float(h0 << 16), r1 = x[1] - __uint_as_float(h0 & 0xffff0000u);
  const float r2 = x[2] - __uint_as_float(h1 << 16), r3 = x[3] - __uint_as_float(h1 & 0xffff0000u);
  const uint32_t l0 = pk_bf16(r0, r1), l1 = pk_bf16(r2, r3);
  const uint2 hv = make_uint2(h0, h1), lv = make_uint2(l0, l1);
  hi = __builtin_bit_cast(s4v, hv);
  lo = __builtin_bit_cast(s4v, lv);
}

template <int KT, typename TI, typename TO, bool F32>
__global__ __launch_bounds__(1024) void harp_stream_mfma_kernel(
    const TI *__restrict__ X, int64_t ldx, TO *__restrict__ Y, int64_t ldy, int64_t n,
    int rows_per_wg, int gx, int gy, PassDesc pd) {
  constexpr bool in_bf16 = sizeof(TI) == 2, out_bf16 = sizeof(TO) == 2;
  constexpr int MAXG = (kRC * 16 * KT * 4 + 1023) / 1024;   // 4-coordinate groups per thread
  __shared__ float tile[16 * KT * kJS];
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave = block within the q tile
  const int l = tid & 63, g = l >> 4, c16 = l & 15;
  const int b = pd.b, S = pd.S;
  // workgroup id -> (q tile qx, row group ry); gx = q tiles, gy = row groups
  int qx, ry;
  if ((gx & 3) == 0) {
    const int xcd = blockIdx.x & 7, i = blockIdx.x >> 3;
    const int unit = (i >> 2) * 8 + xcd;          // (quad of q tiles, row group)
    const int nquad = gx >> 2;
    if (unit >= nquad * gy) return;               // grid padded to a multiple of 32
    qx = (unit % nquad) * 4 + (i & 3);
    ry = unit / nquad;
  } else {
    qx = blockIdx.x % gx;
    ry = blockIdx.x / gx;
  }
  const int q0 = qx * 16;
  const int hi = q0 / S, lo0 = q0 - hi * S;
  const int64_t base = (int64_t)hi * b * S + lo0;
  const int64_t r_begin = (int64_t)ry * rows_per_wg;
  const int64_t r_end = (r_begin + rows_per_wg < n) ? r_begin + rows_per_wg : n;

  // this wave's block, packed by the plan in lane layout: tile (kt, nt), half 0 = hi, 1 = lo;
  // the float32 copy of the same tiles (one float4 per lane and tile) follows the bf16 tiles
  // of all nq blocks
  s4v bh[F32 ? 1 : KT][F32 ? 1 : KT], bl[F32 ? 1 : KT][F32 ? 1 : KT];
  f4v bf[F32 ? KT : 1][F32 ? KT : 1];
  // block of this wave in the plan's packed image (tied parameters: the one shared table)
  const size_t qb = pd.tied ? 0 : (size_t)(q0 + w);
  if constexpr (F32) {
    const f4v *bp = reinterpret_cast<const f4v *>(static_cast<const s4v *>(pd.aux) +
                                                  (size_t)pd.nqp * KT * KT * 2 * 64) +
                    qb * KT * KT * 64 + l;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
      for (int nt = 0; nt < KT; ++nt) bf[kt][nt] = bp[(kt * KT + nt) * 64];
  } else {
    const s4v *bp = static_cast<const s4v *>(pd.aux) + qb * KT * KT * 2 * 64 + l;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
      for (int nt = 0; nt < KT; ++nt) {
        bh[kt][nt] = bp[((kt * KT + nt) * 2 + 0) * 64];
        bl[kt][nt] = bp[((kt * KT + nt) * 2 + 1) * 64];
      }
  }

  const int ngroups = kRC * b * 4;   // (row, j, quarter of the 16 lo) per chunk
  // This thread's 4-coordinate groups: offsets inside a chunk of 16 rows (32-bit) and LDS slots.
  // A thread whose group index lies beyond the chunk takes the group of another thread a second
  // time (same loads, same values to the same LDS slots and addresses), so that inside full
  // chunks no access is conditional.
  unsigned offx[MAXG], offy[MAXG];
  int grow[MAXG], gtile[MAXG];
#pragma unroll
  for (int u = 0; u < MAXG; ++u) {
    const int gi = (tid + u * 1024) % ngroups;
    const int lo4 = gi & 3, rem = gi >> 2;
    const int row = rem & (kRC - 1), j = rem >> 4;
    grow[u] = row;
    offx[u] = (unsigned)(row * (int)ldx + j * S + lo4 * 4);
    offy[u] = (unsigned)(row * (int)ldy + j * S + lo4 * 4);
    gtile[u] = j * kJS + (lo4 * 4) * kLS + row;
  }
  float pre[MAXG][4];
  // rows [r0, r0 + left) of the chunk exist; FULL: left == 16 and nothing is tested
  auto fetch = [&](int64_t r0, int left, auto full) {
    const TI *xc = X + r0 * ldx + base;
#pragma unroll
    for (int u = 0; u < MAXG; ++u) {
      if (!decltype(full)::value) pre[u][0] = pre[u][1] = pre[u][2] = pre[u][3] = 0.0f;
      if (decltype(full)::value || grow[u] < left) {
        if constexpr (in_bf16) {
          const uint2 v = *reinterpret_cast<const uint2 *>(xc + offx[u]);
          pre[u][0] = __uint_as_float(v.x << 16);
          pre[u][1] = __uint_as_float(v.x & 0xffff0000u);
          pre[u][2] = __uint_as_float(v.y << 16);
          pre[u][3] = __uint_as_float(v.y & 0xffff0000u);
        } else {
          const float4 v = *reinterpret_cast<const float4 *>(xc + offx[u]);
          pre[u][0] = v.x; pre[u][1] = v.y; pre[u][2] = v.z; pre[u][3] = v.w;
        }
      }
    }
  };
  auto commit = [&]() {
#pragma unroll
    for (int u = 0; u < MAXG; ++u) {
      float *t = tile + gtile[u];
#pragma unroll
      for (int k = 0; k < 4; ++k) t[k * kLS] = pre[u][k];
    }
  };
  // the chunk in the tile times this wave's block, results back into the same tile positions
  auto multiply = [&]() {
    // ---- A operand: lane (row = c16, k = 4g + i) of this wave's block
    f4v acc[KT];
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) acc[nt] = (f4v){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      float a[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = 16 * kt + 4 * g + i;
        a[i] = (j < b) ? tile[j * kJS + w * kLS + c16] : 0.0f;
      }
      if constexpr (F32) {
        // k = 16 kt + 4 g + i is summed by instruction i: operand lanes (row | column, g)
#pragma unroll
        for (int nt = 0; nt < KT; ++nt)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], bf[kt][nt][i], acc[nt], 0, 0, 0);
      } else {
        s4v ah, al;   // split to bf16 hi/lo
        split4(a, ah, al);
#pragma unroll
        for (int nt = 0; nt < KT; ++nt) {
          acc[nt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(al, bh[kt][nt], acc[nt], 0, 0, 0);
          acc[nt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ah, bl[kt][nt], acc[nt], 0, 0, 0);
          acc[nt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ah, bh[kt][nt], acc[nt], 0, 0, 0);
        }
      }
    }
    __syncthreads();   // every wave has read its inputs
    // ---- lane holds rows 4g..4g+3 of output coordinate 16nt + c16
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
      const int j2 = 16 * nt + c16;
      if (j2 < b) {
        float *t = tile + j2 * kJS + w * kLS + 4 * g;
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = acc[nt][i];
      }
    }
    __syncthreads();
  };
  // coalesced store of the chunk in the tile
  auto put = [&](int64_t r0, int left, auto full) {
    TO *yc = Y + r0 * ldy + base;
#pragma unroll
    for (int u = 0; u < MAXG; ++u) {
      if (decltype(full)::value || grow[u] < left) {
        const float *t = tile + gtile[u];
        const float v0 = t[0], v1 = t[kLS], v2 = t[2 * kLS], v3 = t[3 * kLS];
        if constexpr (out_bf16)
          *reinterpret_cast<uint2 *>(yc + offy[u]) = make_uint2(pk_bf16(v0, v1), pk_bf16(v2, v3));
        else
          *reinterpret_cast<float4 *>(yc + offy[u]) = make_float4(v0, v1, v2, v3);
      }
    }
  };
  const std::true_type kFull;
  const std::false_type kGuarded;

  // Full chunks: the next chunk is requested while this one is computed (after the last one
  // that chunk itself once more), so that the wait for it, before it goes into the tile, always
  // follows this chunk's stores and nothing else: it need not wait for those stores.
  const int nfull = (int)((r_end - r_begin) / kRC);
  const int tail = (int)(r_end - r_begin) - nfull * kRC;
  if (nfull > 0) {
    fetch(r_begin, kRC, kFull);
    commit();
    __syncthreads();
    for (int c = 0; c < nfull; ++c) {
      const int64_t r0 = r_begin + (int64_t)c * kRC;
      fetch((c + 1 < nfull) ? r0 + kRC : r0, kRC, kFull);
      multiply();
      put(r0, kRC, kFull);
      __syncthreads();   // the tile is free again
      commit();
      __syncthreads();
    }
  }
  if (tail > 0) {   // the rows left over at the end of the matrix
    const int64_t r0 = r_begin + (int64_t)nfull * kRC;
    fetch(r0, tail, kGuarded);
    commit();
    __syncthreads();
    multiply();
    put(r0, tail, kGuarded);
  }
}

template <int KT, typename TI, typename TO, bool F32>
harp_status_t launch_mfma_typed(const harp_plan *plan, const PassDesc &pd, const void *X,
                                int64_t ldx, void *Y, int64_t ldy, int64_t n,
                                hipStream_t stream) {
  const unsigned gx = (unsigned)(pd.nq / 16);
  // one workgroup (16 waves) per compute unit and wave of the grid; rows in multiples of 16
  int64_t gy = (plan->num_cu + gx - 1) / gx;
  if (gy < 1) gy = 1;
  int64_t rpw = (n + gy - 1) / gy;
  rpw = ((rpw + kRC - 1) / kRC) * kRC;
  gy = (n + rpw - 1) / rpw;
  int64_t total = (int64_t)gx * gy;
  if ((gx & 3) == 0) total = (total + 31) / 32 * 32;
  if (total > 0x7fffffff) return HARP_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((harp_stream_mfma_kernel<KT, TI, TO, F32>), dim3((unsigned)total), dim3(1024), 0,
                     stream, (const TI *)X, ldx, (TO *)Y, ldy, n, (int)rpw, (int)gx, (int)gy, pd);
  return hipGetLastError() == hipSuccess ? HARP_OK : HARP_ERR_DEVICE;
}

// the streamed stage sits between the caller's bf16 side and the float32 intermediate, or
// between two float32 intermediates
template <int KT>
harp_status_t launch_mfma_inst(const harp_plan *plan, const PassDesc &pd, const void *X,
                               int64_t ldx, int ib, void *Y, int64_t ldy, int ob, int64_t n,
                               bool narrow, hipStream_t stream) {
  if (!narrow) {   // float32 on both sides of the call: every segment is float32
    if (ib || ob) return HARP_ERR_INVALID_ARG;
    return launch_mfma_typed<KT, float, float, true>(plan, pd, X, ldx, Y, ldy, n, stream);
  }
  if (ib && !ob)
    return launch_mfma_typed<KT, uint16_t, float, false>(plan, pd, X, ldx, Y, ldy, n, stream);
  if (!ib && ob)
    return launch_mfma_typed<KT, float, uint16_t, false>(plan, pd, X, ldx, Y, ldy, n, stream);
  if (!ib && !ob)
    return launch_mfma_typed<KT, float, float, false>(plan, pd, X, ldx, Y, ldy, n, stream);
  return launch_mfma_typed<KT, uint16_t, uint16_t, false>(plan, pd, X, ldx, Y, ldy, n, stream);
}

}  // namespace

bool mfma_pass_supported(const PassDesc &pd, const void *X, int64_t ldx, const void *Y,
                         int64_t ldy) {
  if (pd.kind != PASS_GENERIC || pd.b < 9 || pd.b > 64 || pd.aux == nullptr) return false;
  if (pd.S % 16 != 0) return false;   // 16 consecutive blocks must be 16 consecutive coordinates
  if ((ldx % 4) || (ldy % 4) || ((uintptr_t)X % 16) || ((uintptr_t)Y % 16)) return false;
  if (ldx >= ((int64_t)1 << 26) || ldy >= ((int64_t)1 << 26)) return false;   // 32-bit offsets per chunk
  return true;
}

harp_status_t launch_mfma_pass(const harp_plan *plan, const PassDesc &pd, const void *X,
                               int64_t ldx, harp_dtype_t dt_in, void *Y, int64_t ldy,
                               harp_dtype_t dt_out, int64_t n, bool narrow, hipStream_t stream) {
  if (n == 0) return HARP_OK;
  const int ib = dt_in == HARP_BF16, ob = dt_out == HARP_BF16;
  const int kt = (pd.b + 15) / 16;
  switch (kt) {
    case 1: return launch_mfma_inst<1>(plan, pd, X, ldx, ib, Y, ldy, ob, n, narrow, stream);
    case 2: return launch_mfma_inst<2>(plan, pd, X, ldx, ib, Y, ldy, ob, n, narrow, stream);
    case 3: return launch_mfma_inst<3>(plan, pd, X, ldx, ib, Y, ldy, ob, n, narrow, stream);
    case 4: return launch_mfma_inst<4>(plan, pd, X, ldx, ib, Y, ldy, ob, n, narrow, stream);
    default: return HARP_ERR_UNSUPPORTED;
  }
}

}  // namespace harp
