// C ABI of libharp: plan construction (validation, pass grouping, parameter packing),
// dispatch of apply / apply_transpose / rotate_weight, helpers.  Host code only; the
// kernels and their launchers are in harp_kernels.hip.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "harp_internal.h"

using namespace harp;

// Intermediate of harp_apply_noalloc: device memory that belongs to the loaded library, one copy
// per GPU, held until the process ends.  In host code the name stands for the symbol, not for
// a device address: the address is looked up once per device (noalloc_scratch below) and only
// that pointer is ever handed to a kernel.
#define HARP_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
static __device__ __align__(256) float scratch[HARP_NOALLOC_SCRATCH_BYTES / sizeof(float)];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_noalloc_mu;
float *g_noalloc_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up at the first call on it).
harp_status_t noalloc_scratch(int dev, float **out) {
  if (dev < 0 || dev >= kMaxDevices) return HARP_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_noalloc_mu);
  if (!g_noalloc_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return HARP_ERR_DEVICE;
    }
    g_noalloc_ptr[dev] = (float *)p;
  }
  *out = g_noalloc_ptr[dev];
  return HARP_OK;
}

// Effective form of one executed stage (a direction's program), after the +-1 signs of the
// processor and the signs released by earlier lifted stages have been folded in.
//
// A 2x2 orthogonal block M (row vector on the left) factors as R * diag(d0, d1) with
// R = [[C, -S], [S, C]], C >= 0, and R as three shears (lifting steps)
//     x0 += a x1;  x1 += b x0;  x0 += a x1;      a = S / (1 + C),  b = -S,
// which costs 3 fused multiply-adds per coordinate pair instead of 4 operations, with
// |a|, |b| <= 1.  The output signs d0, d1 are not applied: they are pushed onto the input rows
// of whichever later stage touches those coordinates.  A dense stage absorbs all pending
// signs into the rows of its blocks.  The last stage of a program is always dense and also
// takes the processor's output signs (transposed direction) on its columns, so no kernel
// ever multiplies by a sign vector.
//
// Cheaper still, and the form tried first: any 2x2 block M = [[m00, m01], [m10, m11]] with a
// non-zero diagonal factors as
//     y0 = m00 (x0 + (m10 / m00) x1),     y1 = m11 (x1 + (m01 / m11) x0),
// two independent fused multiply-adds per pair; the output scales m00, m11 are not applied
// but pushed, like the signs above, onto the rows of whichever later stage touches the
// coordinate (so a coordinate travels divided by a known scale until a dense stage - at the
// latest the program's last - multiplies it back in).  The arithmetic is that of the dense
// product carried out in scaled units, so rounding errors stay relative to the same
// quantities.  A program takes this form only if every pending scale stays within
// [2^-60, 2^60] and every shear factor within 2^40 in magnitude (no overflow for |x| < 2^64);
// otherwise it falls back to lifting.
enum StageForm { FORM_DENSE = 0, FORM_LIFT = 1, FORM_SCALED = 2 };

struct StageEff {
  int t = 0;
  int32_t b = 0;
  int64_t s = 0;
  int form = FORM_DENSE;
  std::vector<float> dense;   // [D][b][b], E'[c][r][r2]            (FORM_DENSE)
  std::vector<float> la, lb;  // [D] lifting coefficients (a, b) or shear factors (m10/m00, m01/m11)
};

inline int64_t coord_of(int64_t c, int r, int32_t b, int64_t s) {
  const int64_t alpha = c / s, beta = c % s;   // Lemma 1: alpha*b*s + r*s + beta
  return alpha * b * s + (int64_t)r * s + beta;
}

// true when every 2x2 block is a rotation or a reflection to float32 rounding
bool stage_orthogonal_2x2(const float *K, int64_t D) {
  for (int64_t c = 0; c < D; ++c) {
    const double e00 = K[c * 4 + 0], e01 = K[c * 4 + 1], e10 = K[c * 4 + 2], e11 = K[c * 4 + 3];
    if (std::fabs(e00 * e00 + e10 * e10 - 1.0) > 4e-7) return false;
    const double rot = std::fabs(e01 + e10) + std::fabs(e11 - e00);   // [[c,-s],[s,c]]
    const double ref = std::fabs(e01 - e10) + std::fabs(e11 + e00);   // [[c, s],[s,-c]]
    if (std::min(rot, ref) > 3e-7) return false;
  }
  return true;
}

// scaled == true: radix-2 stages before the last take the two-shear form; returns false when a
// block has a (near-)zero diagonal or a pending scale leaves the safe range.
// dense_t >= 0: stage dense_t of a forward program is kept dense although it is not the last
// (the end of the slices of a plan with tied parameters; the end of the chunk whose output
// travels as block-scaled halves), so that no scale is pending behind it.
bool build_effective(const harp_plan *plan, const std::vector<const float *> &blocks,
                     const int8_t *signs, int algo, Direction dir, bool scaled,
                     std::vector<StageEff> &out, int dense_t = -1, int dense_both = -1) {
  const int m = plan->m;
  const int64_t d = plan->d;
  const double kScaleMax = 1152921504606846976.0;   // 2^60
  std::vector<double> tau(d, 1.0);
  if (dir == DIR_FWD && signs)
    for (int64_t i = 0; i < d; ++i) tau[i] = (double)signs[i];
  out.clear();
  out.resize(m);
  for (int i = 0; i < m; ++i) {
    const int t = (dir == DIR_FWD) ? i : m - 1 - i;
    StageEff &se = out[i];
    se.t = t;
    se.b = plan->radices[t];
    se.s = plan->strides[t];
    const int b = se.b;
    const int64_t D = d / b;
    const float *K = blocks[t];
    const bool last = (i == m - 1);
    auto E = [&](int64_t c, int r, int r2) -> double {   // block as used in this direction
      return dir == DIR_TRN ? K[(c * b + r2) * b + r] : K[(c * b + r) * b + r2];
    };
    // Tied parameters, forward: the last stage of the slices is dense as well, so that no
    // pending scale (a function of the coordinate inside the slice) reaches the table, whose
    // blocks then really are one matrix.  Likewise the last stage of a chunk whose output is
    // stored as block-scaled halves: those need values of the row's own size.
    // (dense_both: a radix-2 stage streamed on its own above the chunk, with the halves on one side
    // of it in either direction)
    const bool slice_end = (dir == DIR_FWD && t == dense_t) || t == dense_both;
    const bool pow2_stage = (algo != HARP_ALGO_GENERIC && b == 2 && !last && !slice_end);
    if (pow2_stage && scaled) {
      se.form = FORM_SCALED;
      se.la.resize(D);
      se.lb.resize(D);
      for (int64_t c = 0; c < D; ++c) {
        const int64_t i0 = coord_of(c, 0, 2, se.s), i1 = coord_of(c, 1, 2, se.s);
        const double m00 = tau[i0] * E(c, 0, 0), m01 = tau[i0] * E(c, 0, 1);
        const double m10 = tau[i1] * E(c, 1, 0), m11 = tau[i1] * E(c, 1, 1);
        const double a0 = std::fabs(m00), a1 = std::fabs(m11);
        if (!(a0 >= 1.0 / kScaleMax && a0 <= kScaleMax && a1 >= 1.0 / kScaleMax &&
              a1 <= kScaleMax))
          return false;
        const float f0 = (float)(m10 / m00), f1 = (float)(m01 / m11);
        // |shear factor| <= 2^40: with scales >= 2^-60 the sheared values of |x| < 2^64 stay finite
        if (!(std::fabs(f0) <= 1099511627776.0f) || !(std::fabs(f1) <= 1099511627776.0f)) return false;
        se.la[c] = f0;
        se.lb[c] = f1;
        tau[i0] = m00;
        tau[i1] = m11;
      }
      continue;
    }
    se.form = (pow2_stage && stage_orthogonal_2x2(K, D)) ? FORM_LIFT : FORM_DENSE;
    if (se.form == FORM_LIFT) {
      se.la.resize(D);
      se.lb.resize(D);
      for (int64_t c = 0; c < D; ++c) {
        const int64_t i0 = coord_of(c, 0, 2, se.s), i1 = coord_of(c, 1, 2, se.s);
        const double m00 = tau[i0] * E(c, 0, 0), m01 = tau[i0] * E(c, 0, 1);
        const double m10 = tau[i1] * E(c, 1, 0), m11 = tau[i1] * E(c, 1, 1);
        const double d0 = (m00 >= 0.0) ? 1.0 : -1.0;
        const double C = d0 * m00, S = d0 * m10;
        const double d1 = (m11 * C - m01 * S >= 0.0) ? 1.0 : -1.0;
        se.la[c] = (float)(S / (1.0 + C));
        se.lb[c] = (float)(-S);
        tau[i0] = d0;
        tau[i1] = d1;
      }
    } else {
      se.dense.resize((size_t)D * b * b);
      for (int64_t c = 0; c < D; ++c) {
        for (int r = 0; r < b; ++r) {
          const int64_t ir = coord_of(c, r, b, se.s);
          for (int r2 = 0; r2 < b; ++r2) {
            double v = tau[ir] * E(c, r, r2);
            if (last && dir == DIR_TRN && signs) v *= (double)signs[coord_of(c, r2, b, se.s)];
            se.dense[((size_t)c * b + r) * b + r2] = (float)v;
          }
        }
        for (int r = 0; r < b; ++r) tau[coord_of(c, r, b, se.s)] = 1.0;
      }
    }
  }
  return true;
}

constexpr int64_t kChunkCap = 4096;   // largest on-chip chunk of a split program
constexpr int kChainMax = 2;          // radix-3 stages per streamed trip

// Split a run of `len` stages into ceil(len / kmax) nearly equal parts.
void split_run(int len, int kmax, std::vector<int> &out) {
  int parts = (len + kmax - 1) / kmax;
  int base = len / parts, extra = len % parts;
  for (int i = 0; i < parts; ++i) out.push_back(base + (i < extra ? 1 : 0));
}

int ilog2(int64_t v) {
  int l = 0;
  while ((int64_t(1) << l) < v) ++l;
  return l;
}

// Build the pass list and the packed parameter image for one (algo, direction).
// Layout of the image: per pass, V rows of nq floats (value v of sub-tensor q at v*nq + q),
// so that consecutive threads (consecutive q) read consecutive addresses.
uint16_t bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
float bf16_to_float(uint16_t h) {
  const uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

// A radix-b block (9 <= b <= 64) as operand tiles of v_mfma_f32_16x16x16_bf16: KT = ceil(b/16);
// for tile (kt, nt), half h (0: bf16(v), 1: bf16(v - hi)), lane l, i < 4 the value is
// K[k = 16 kt + 4 (l / 16) + i][n = 16 nt + l % 16], zero outside the block.  out32 takes the
// same tiles unsplit in float32, [tile][lane][i], for v_mfma_f32_16x16x4_f32 (instruction i of
// a tile sums the four k of index i).
void pack_mfma_block(const float *K, int b, uint16_t *out, float *out32) {
  const int KT = (b + 15) / 16;
  for (int kt = 0; kt < KT; ++kt)
    for (int nt = 0; nt < KT; ++nt)
      for (int l = 0; l < 64; ++l)
        for (int i = 0; i < 4; ++i) {
          const int k = 16 * kt + 4 * (l / 16) + i, n = 16 * nt + l % 16;
          const float v = (k < b && n < b) ? K[k * b + n] : 0.0f;
          const uint16_t hi = bf16_rne(v);
          const uint16_t lo = bf16_rne(v - bf16_to_float(hi));
          const size_t t = (size_t)(kt * KT + nt) * 2;
          out[((t + 0) * 64 + l) * 4 + i] = hi;
          out[((t + 1) * 64 + l) * 4 + i] = lo;
          out32[((size_t)(kt * KT + nt) * 64 + l) * 4 + i] = v;
        }
}

// Image of the two-group DPP kernel for the chunk-local stages of a program: exactly twelve
// radix-2 stages on the digits 0..11 (ascending in a forward program, descending in a
// transposed one), all in the two-shear form except that the last may be the program's dense
// last stage.  eff[i0 .. i0 + 12) are those stages in execution order.  Appends to `image`.
void build_dpp_image(const harp_plan *plan, const std::vector<StageEff> &eff, int i0, Direction dir,
                     HostProgram &hp, std::vector<float> &image, int dense_i = -1, int L = 12) {
  const int D = 1 << L, TG = D / 16;   // L = 12, or 11 (chunks of 2048, 128 threads per group)
  hp.dpp = DppImage();
  const int m = plan->m;
  if (i0 < 0 || i0 + L > m || plan->d % D) return;
  bool ld = false;
  for (int e = 0; e < L; ++e) {
    const StageEff &se = eff[i0 + e];
    const int digit = (dir == DIR_FWD) ? e : L - 1 - e;
    if (se.b != 2 || se.s != ((int64_t)1 << digit)) return;
    if (se.form == FORM_SCALED) continue;
    // (dense_i: the chunk's last stage kept dense in a forward split program, see build_program)
    if (se.form == FORM_DENSE && e == L - 1 && (i0 + e == m - 1 || i0 + e == dense_i)) {
      ld = true;
      continue;
    }
    return;
  }
  if (dir == DIR_TRN && !ld) return;
  const bool trn = (dir == DIR_TRN);
  const int nsa = trn ? L - 8 : 8;             // shear stages of group A
  const int nsb = L - nsa - (ld ? 1 : 0);      // shear stages of group B
  const int64_t nchunk = plan->d / D;
  const int64_t strideA = (int64_t)nsa * D, strideB = (int64_t)(nsb + (ld ? 2 : 0)) * D;
  const size_t off = image.size();
  image.resize(off + (size_t)nchunk * (strideA + strideB));
  float *base = image.data() + off;
  // factor of global coordinate i in execution stage e: the member with digit value 0 holds
  // m10 / m00 (it receives the other member), the member with digit value 1 holds m01 / m11
  auto block_of = [&](const StageEff &se, int64_t i) { return (i / (2 * se.s)) * se.s + i % se.s; };
  for (int64_t kch = 0; kch < nchunk; ++kch)
    for (int grp = 0; grp < 2; ++grp) {
      // group A works in the low layout going up and in the high layout going down; B the other
      const bool high = (grp == 0) ? trn : !trn;
      float *g = base + (grp == 0 ? kch * strideA : nchunk * strideA + kch * strideB);
      const int e0 = grp == 0 ? 0 : nsa, ne = grp == 0 ? nsa : nsb + (ld ? 1 : 0);
      for (int ee = 0; ee < ne; ++ee) {
        const StageEff &se = eff[i0 + e0 + ee];
        const bool dense = (se.form == FORM_DENSE);
        for (int k = 0; k < 4; ++k)
          for (int t = 0; t < TG; ++t)
            for (int q = 0; q < 4; ++q) {
              const int64_t i = kch * D + 16 * (int64_t)dpp_segment_of(high, (unsigned)t, L) + 4 * k + q;
              const int64_t c = block_of(se, i);
              const int r = (int)((i / se.s) & 1);
              const size_t slot = ((size_t)(ee * 4 + k) * TG + t) * 4 + q;
              if (!dense) {
                g[slot] = r == 0 ? se.la[c] : se.lb[c];
              } else {
                // y_r = x_r E[r][r] + x_(1-r) E[1-r][r]
                g[slot] = se.dense[(size_t)c * 4 + r * 2 + r];
                g[slot + (size_t)D] = se.dense[(size_t)c * 4 + (1 - r) * 2 + r];
              }
            }
      }
    }
  hp.dpp.host_off = (int64_t)off;
  hp.dpp.offB = nchunk * strideA;
  hp.dpp.strideA = strideA;
  hp.dpp.strideB = strideB;
  hp.dpp.trn = trn;
  hp.dpp.ld = ld;
  hp.dpp.logd = L;
}

bool build_program(const harp_plan *plan, const std::vector<const float *> &blocks,
                   const int8_t *signs, int algo, Direction dir, HostProgram &hp,
                   std::vector<float> &image, std::vector<size_t> &offsets,
                   std::vector<std::vector<uint16_t>> &aux) {
  const int m = plan->m;
  const int64_t d = plan->d;
  // A plan with tied parameters has the split program only; its signs are applied by the wave
  // kernel (folded into the stage parameters they would make every slice's image different).
  const bool tied = plan->tied_K > 0;
  if (tied && algo != HARP_ALGO_SPLIT) return false;
  if (tied) signs = nullptr;

  Program &pg = hp.prog;
  pg.npass = 0;
  image.clear();
  offsets.clear();
  aux.assign(kMaxPasses, std::vector<uint16_t>());

  // Split programs: stages t < tb (product of their radices = chunk <= kChunkCap, maximal unless
  // a large-radix stage ends it earlier) are chunk-local; passes never mix stages from both
  // sides of tb.
  const bool fused = (algo != HARP_ALGO_GENERIC);
  int tb = m;
  int64_t chunk = d;
  if (algo == HARP_ALGO_SPLIT) {
    tb = 0;
    chunk = 1;
    bool small_only = true;   // every stage of the chunk so far has radix <= 8
    while (tb < m && chunk * plan->radices[tb] <= kChunkCap) {
      // A stage of radix >= 9 that the matrix-core kernel can stream (its stride, the chunk so
      // far, a multiple of 16) ends a chunk of small-radix stages: on chip such a stage only
      // has the run-time-radix body, which re-reads its block for every row.
      const bool large = plan->radices[tb] >= 9;
      if (large && small_only && chunk >= 64 && chunk % 16 == 0) break;
      if (large) small_only = false;
      chunk *= plan->radices[tb++];
    }
    // A chunk of radix-2 stages followed by other small radices has no kernel of its own (the
    // pipelined and wave kernels take radix-2 chains, the radix kernels radices 3..8): end it
    // behind the radix-2 stages when those alone make a chunk of 256 or more, and stream the
    // rest (13824 = 2^9 * 27, n = 2048: 193 -> 136 us).  Only for rows longer than the cap: up
    // to 4096 the one-launch tile kernel measured as fast or faster (2304 .. 3840 with tails
    // of radix 5, 7, 3*3, 3*5; every transposed program; and 3 us less at small batch sizes).
    int t2 = 0;
    while (t2 < tb && plan->radices[t2] == 2) ++t2;
    // [2 .. 2, 3] up to 4096 (768, 1536, 3072): kept as a second program for large forward
    // batches (n = 2048: 19 -> 12, 21.5 -> 16.3, 27.9 -> 23.2 us).
    const bool tail3 = (d <= kChunkCap && t2 == m - 1 && plan->radices[m - 1] == 3);
    if ((d > kChunkCap || tail3) && t2 < tb && t2 >= 8 && small_only) {
      tb = t2;
      chunk = (int64_t)1 << t2;
      hp.optional = tail3;
    }
    if (tb == 0 || tb == m) return false;   // nothing to split: the fused program covers it
    // tied: the chunk is exactly one slice, the table is the one streamed stage (matrix cores)
    if (tied && (chunk != plan->tied_n2 || tb != m - 1 || plan->radices[m - 1] < 9)) return false;
  }
  // Block-scaled half intermediate (bf16 callers): one streamed stage of radix >= 3 (dense in
  // both directions, so nothing is pending behind it going down), orthogonal blocks, and a
  // dense stage at the end of the chunk going up.
  // (only where both kernels of the pair handle the format: chunks of 4096 on the DPP kernel or
  // of 256 / 512 / 1024 on the wave kernel, and the small-radix streamed kernel)
  bool tops_small = (tb < m);   // every streamed stage of radix 3..8
  for (int t = tb; t < m; ++t) tops_small = tops_small && plan->radices[t] >= 3 && plan->radices[t] <= 8;
  // ... or one radix-2 stage on the top digit (8192 = 2^13): kept dense in both directions, it is
  // streamed by the same kernels as a radix-2 "small" stage
  const bool top2 = (algo == HARP_ALGO_SPLIT && !tied && tb == m - 1 && plan->radices[m - 1] == 2);
  tops_small = tops_small || top2;
  hp.z16 = (algo == HARP_ALGO_SPLIT && !tied && plan->orthogonal && !plan->f32_only && tops_small && d % 64 == 0 &&
            (chunk == 4096 || chunk == 2048 || chunk == 1024 || chunk == 512 || chunk == 256));
  const int dense_t = tied ? m - 2 : ((hp.z16 && plan->radices[tb - 1] == 2) ? tb - 1 : -1);
  std::vector<StageEff> eff;
  const int dense_both = (top2 && hp.z16) ? m - 1 : -1;
  if (!build_effective(plan, blocks, signs, algo, dir, true, eff, dense_t, dense_both)) {
    if (tied) return false;
    build_effective(plan, blocks, signs, algo, dir, false, eff, dense_t, dense_both);
  }
  auto local = [&](int i) { return eff[i].t < tb; };
  hp.chunk = (int32_t)chunk;
  hp.n_chunk = 0;
  hp.chunk_first = (dir == DIR_FWD);

  int i = 0;
  while (i < m) {
    const int b = eff[i].b;
    if (fused && b == 2) {
      // sub-run of radix-2 stages of one form (and one side of tb); a lifted sub-run may end
      // with the program's final (dense) stage
      const int form = eff[i].form;
      const bool lift = (form != FORM_DENSE);   // two values per pair: lifting or scaled shears
      int len = 1;
      while (i + len < m && eff[i + len].b == 2 && eff[i + len].form == form &&
             local(i + len) == local(i))
        ++len;
      bool last_dense = false;
      // (tied parameters, forward: the dense stage that ends the slices, see build_effective)
      const int dense_at = (dense_t >= 0 && dir == DIR_FWD) ? dense_t : m - 1;
      if (lift && i + len == dense_at && eff[dense_at].b == 2 && eff[dense_at].form == FORM_DENSE &&
          local(dense_at) == local(i)) {
        ++len;
        last_dense = true;
      }
      std::vector<int> parts;
      split_run(len, lift ? 4 : 3, parts);
      // Ten stages split (4, 3, 3).  In a transposed program the digits run downwards, so the
      // pass on the four lowest digits -- the one whose layout is 16 consecutive coordinates
      // per thread, in which the wave kernel can store without a further exchange -- has to
      // come last: (3, 3, 4).
      if (dir == DIR_TRN && lift && len == 10 && local(i) && chunk == 1024)
        std::reverse(parts.begin(), parts.end());
      for (size_t pi = 0; pi < parts.size(); ++pi) {
        const int k = parts[pi];
        const bool ld = last_dense && pi + 1 == parts.size();
        if (pg.npass >= kMaxPasses) return false;
        PassDesc &pd = pg.pass[pg.npass++];
        if (local(i)) ++hp.n_chunk;
        const int P = 1 << k;
        int64_t S = eff[i].s;
        for (int e = 0; e < k; ++e) S = std::min<int64_t>(S, eff[i + e].s);
        const int64_t nq = d / P;
        const int64_t nqp = tied ? chunk / P : nq;   // sub-tensors in the image
        if (tied && (!local(i) || form != FORM_SCALED)) return false;
        if (form == FORM_SCALED)
          pd.kind = ld ? PASS_POW2_SCALED_LD : PASS_POW2_SCALED;
        else
          pd.kind = lift ? (ld ? PASS_POW2_LIFT_LD : PASS_POW2_LIFT) : PASS_POW2_DENSE;
        pd.b = 2;
        pd.k = k;
        pd.desc = (dir == DIR_TRN) ? 1 : 0;
        pd.P = P;
        pd.S = (int32_t)S;
        pd.nq = (int32_t)nq;
        pd.nqp = (int32_t)nqp;
        pd.tied = tied ? 1 : 0;
        pd.V = lift ? (ld ? (k + 1) * P : k * P) : k * (P / 2) * 4;
        offsets.push_back(image.size());
        image.resize(image.size() + (size_t)pd.V * nqp);
        float *img = image.data() + offsets.back();
        for (int e = 0; e < k; ++e) {
          const StageEff &se = eff[i + e];
          const int bp = ilog2(se.s / S);
          // the kernels assume digit position e (ascending) or k-1-e (descending)
          if (bp != (pd.desc ? k - 1 - e : e)) return false;
          for (int64_t q = 0; q < nqp; ++q) {
            const int64_t hi = q / S, lo = q % S;
            const int64_t base = hi * P * S + lo;
            for (int p = 0; p < P / 2; ++p) {
              const int j0 = ((p >> bp) << (bp + 1)) | (p & ((1 << bp) - 1));
              const int64_t idx0 = base + (int64_t)j0 * S;
              const int64_t beta = idx0 % se.s, alpha = idx0 / (2 * se.s);
              const int64_t c = alpha * se.s + beta;
              if (se.form != FORM_DENSE) {
                const size_t v0 = (size_t)(e * (P / 2) + p) * 2;
                img[(v0 + 0) * nqp + q] = se.la[c];
                img[(v0 + 1) * nqp + q] = se.lb[c];
              } else {
                // dense 2x2: inside a lifted pass it follows k-1 lifted stages of P values each
                const size_t v0 = lift ? (size_t)(k - 1) * P + (size_t)p * 4
                                       : (size_t)(e * (P / 2) + p) * 4;
                for (int w = 0; w < 4; ++w) img[(v0 + w) * nqp + q] = se.dense[(size_t)c * 4 + w];
              }
            }
          }
        }
        i += k;
      }
      continue;
    }
    if (pg.npass >= kMaxPasses) return false;
    if (b > HARP_MAX_RADIX) return false;
    // Streamed part of a split program: two consecutive radix-3 stages make one trip through
    // device memory instead of one each (13824 = 2^9 * 27: three trips become two).
    if (fused && b == 3 && !local(i)) {
      int kc = 1;
      while (kc < kChainMax && i + kc < m && eff[i + kc].b == 3 && !local(i + kc) &&
             (eff[i + kc].s == eff[i + kc - 1].s * 3 || eff[i + kc].s * 3 == eff[i + kc - 1].s) &&
             (kc == 1 || ((eff[i + kc].s > eff[i + kc - 1].s) == (eff[i + 1].s > eff[i].s))))
        ++kc;
      if (kc >= 2) {
        PassDesc &pc = pg.pass[pg.npass++];
        const bool desc = eff[i + 1].s < eff[i].s;
        int P = 1;
        for (int e = 0; e < kc; ++e) P *= 3;
        int64_t S = eff[i].s;
        for (int e = 0; e < kc; ++e) S = std::min<int64_t>(S, eff[i + e].s);
        const int NB = P / 3;
        const int64_t nq = d / P;
        pc.kind = PASS_SMALL_CHAIN;
        pc.b = 3;
        pc.k = kc;
        pc.desc = desc ? 1 : 0;
        pc.P = P;
        pc.S = (int32_t)S;
        pc.nq = (int32_t)nq;
        pc.nqp = (int32_t)nq;
        pc.tied = 0;
        pc.V = kc * NB * 9;
        offsets.push_back(image.size());
        image.resize(image.size() + (size_t)pc.V * nq);
        float *img = image.data() + offsets.back();
        for (int64_t q = 0; q < nq; ++q) {
          const int64_t hi = q / S, lo = q % S;
          const int64_t base = hi * P * S + lo;
          for (int k = 0; k < kc; ++k) {
            const StageEff &se = eff[i + k];   // execution order
            int pdig = 0;                      // its digit inside the sub-tensor
            for (int64_t t = S; t < se.s; t *= 3) ++pdig;
            int sp = 1;
            for (int e = 0; e < pdig; ++e) sp *= 3;
            for (int o = 0; o < NB; ++o) {
              const int j0 = (o / sp) * sp * 3 + o % sp;
              const int64_t i0 = base + (int64_t)j0 * S;
              const int64_t c = (i0 / (3 * se.s)) * se.s + i0 % se.s;
              for (int v = 0; v < 9; ++v)
                img[(size_t)((k * NB + o) * 9 + v) * nq + q] = se.dense[(size_t)c * 9 + v];
            }
          }
        }
        i += kc;
        continue;
      }
    }
    PassDesc &pd = pg.pass[pg.npass++];
    if (local(i)) ++hp.n_chunk;
    const bool small = (fused && b >= 3 && b <= 8);
    const StageEff &se = eff[i];
    const int64_t nq = d / b;
    pd.kind = small ? PASS_SMALL : PASS_GENERIC;
    pd.b = b;
    pd.k = 1;
    pd.desc = 0;
    pd.P = b;
    pd.S = (int32_t)se.s;
    if (tied && (local(i) || b < 9)) return false;   // tied: only the table is streamed
    const int64_t nqp = tied ? 1 : nq;
    pd.nq = (int32_t)nq;
    pd.nqp = (int32_t)nqp;
    pd.tied = tied ? 1 : 0;
    pd.V = b * b;
    offsets.push_back(image.size());
    image.resize(image.size() + (size_t)pd.V * nqp);
    float *img = image.data() + offsets.back();
    // sub-tensor q = hi*S + lo is exactly block c = alpha*s + beta with alpha = hi, beta = lo
    for (int64_t q = 0; q < nqp; ++q)
      for (int r = 0; r < b; ++r)
        for (int r2 = 0; r2 < b; ++r2)
          img[(size_t)(r * b + r2) * nqp + q] = se.dense[((size_t)q * b + r) * b + r2];
    if (small && (b == 4 || b == 8)) {
      // second copy for the equal-radix tile kernel, four values per 16-byte load:
      // value v = 4 * v4 + i of sub-tensor q at float index ((v4 * nq) + q) * 4 + i
      std::vector<uint16_t> &a = aux[pg.npass - 1];
      a.resize((size_t)pd.V * nq * 2);
      float *a4 = reinterpret_cast<float *>(a.data());
      for (int64_t q = 0; q < nq; ++q)
        for (int v = 0; v < pd.V; ++v)
          a4[((size_t)(v >> 2) * nq + q) * 4 + (v & 3)] = img[(size_t)v * nq + q];
    }
    if (fused && !small && b >= 9) {   // matrix-core operand tiles for the streamed large radix
      const int KT = (b + 15) / 16;
      const size_t per = (size_t)KT * KT * 2 * 64 * 4;   // bf16 values per block
      const size_t per32 = (size_t)KT * KT * 64 * 4;     // float32 values per block
      std::vector<uint16_t> &a = aux[pg.npass - 1];
      a.resize(per * nqp + 2 * per32 * nqp);             // [nqp] bf16 tiles, then [nqp] float32 tiles
      float *a32 = reinterpret_cast<float *>(a.data() + per * nqp);
      for (int64_t q = 0; q < nqp; ++q)
        pack_mfma_block(se.dense.data() + (size_t)q * b * b, b, a.data() + per * q,
                        a32 + per32 * q);
    }
    ++i;
  }
  hp.param_bytes = (int64_t)image.size() * 4;
  // second image of the same chunk-local stages for the two-group DPP kernel (chunks of 4096)
  hp.dpp = DppImage();
  if (algo == HARP_ALGO_FUSED && chunk == 4096 && tb == 12 && m == 12)
    build_dpp_image(plan, eff, 0, dir, hp, image);
  if (algo == HARP_ALGO_FUSED && chunk == 2048 && tb == 11 && m == 11)
    build_dpp_image(plan, eff, 0, dir, hp, image, -1, 11);
  if (algo == HARP_ALGO_FUSED && chunk == 1024 && tb == 10 && m == 10)
    build_dpp_image(plan, eff, 0, dir, hp, image, -1, 10);
  // Split programs whose intermediate may travel as block-scaled halves: the chunks of 4096 of a
  // bf16 caller run on the DPP kernel too (a thread's 16 coordinates are one segment of that
  // format in both of its layouts).
  if (algo == HARP_ALGO_SPLIT && hp.z16 && chunk == 4096 && tb == 12 && m == 13 &&
      !(dir == DIR_TRN && (eff[0].b == 2 || eff[0].b == 3 || eff[0].b == 5)))   // (those: the image built below)
    build_dpp_image(plan, eff, dir == DIR_FWD ? 0 : 1, dir, hp, image, dir == DIR_FWD ? dense_t : -1);
  const bool top_one_launch = (dir == DIR_TRN && (eff[0].b == 2 || eff[0].b == 3 || eff[0].b == 5));
  if (algo == HARP_ALGO_SPLIT && hp.z16 && chunk == 2048 && tb == 11 && m == 12 && !top_one_launch)
    build_dpp_image(plan, eff, dir == DIR_FWD ? 0 : 1, dir, hp, image, dir == DIR_FWD ? dense_t : -1, 11);
  if (algo == HARP_ALGO_SPLIT && hp.z16 && chunk == 1024 && tb == 10 && m == 11 && !top_one_launch)
    build_dpp_image(plan, eff, dir == DIR_FWD ? 0 : 1, dir, hp, image, dir == DIR_FWD ? dense_t : -1, 10);
  // Transposed split program of ten, eleven or twelve radix-2 stages below one dense stage of radix
  // 2, 3 or 5 (5120, 6144, 10240, 8192, 12288, 20480; radix 7 measured no gain): that stage runs first and is executed by the DPP kernel's first
  // group on the way in (harp_dpp_top_kernel).  Its factors: for output chunk kch, input chunk
  // j and coordinate c of the chunk, entry [j][kch] of block c as this direction uses it.
  if (algo == HARP_ALGO_SPLIT && dir == DIR_TRN && !tied &&
      (chunk == 4096 || chunk == 2048 || chunk == 1024) && chunk == ((int64_t)1 << tb) && m == tb + 1 &&
      (eff[0].b == 2 || eff[0].b == 3 || eff[0].b == 5) && eff[0].form == FORM_DENSE &&
      eff[0].s == chunk && d == chunk * (int64_t)eff[0].b) {
    const int L = tb, TG = (int)(chunk / 16);
    build_dpp_image(plan, eff, 1, dir, hp, image, -1, L);
    if (hp.dpp.host_off >= 0) {
      const int b = eff[0].b;
      const size_t off = image.size();
      image.resize(off + (size_t)b * b * chunk);
      float *tp = image.data() + off;
      for (int kch = 0; kch < b; ++kch)
        for (int j = 0; j < b; ++j)
          for (int k = 0; k < 4; ++k)
            for (int t = 0; t < TG; ++t)
              for (int q = 0; q < 4; ++q) {
                const int64_t c = 16 * (int64_t)dpp_segment_of(true, (unsigned)t, L) + 4 * k + q;
                tp[((((size_t)kch * b + j) * 4 + k) * TG + t) * 4 + q] =
                    eff[0].dense[((size_t)c * b + j) * b + kch];
              }
      hp.dpp.topB = b;
      hp.dpp.offT = (int64_t)off - hp.dpp.host_off;
    }
  }
  hp.ok = true;
  return true;
}

harp_status_t check_apply_args(const harp_plan_t *plan, const void *X, int64_t ldx, const void *Y,
                               int64_t ldy, int64_t n, harp_dtype_t dt) {
  if (!plan) return HARP_ERR_INVALID_ARG;
  if (n < 0) return HARP_ERR_INVALID_ARG;
  if (dt != HARP_F32 && dt != HARP_BF16) return HARP_ERR_INVALID_ARG;
  if (n == 0) return HARP_OK;
  if (!X || !Y) return HARP_ERR_INVALID_ARG;
  if (ldx < plan->d || ldy < plan->d) return HARP_ERR_INVALID_ARG;
  return HARP_OK;
}

size_t esize(harp_dtype_t dt) { return dt == HARP_BF16 ? 2 : 4; }

// Rows of one slab of a split program's float32 intermediate: 128 MB (the measured optimum of
// 32 .. 512 MB on the 14336 / 28672 shapes), a multiple of 256 rows when that many fit.
int64_t slab_rows_cap(int64_t d) {
  int64_t slab = ((int64_t)128 << 20) / (d * 4);
  if (slab >= 512) slab = (slab / 256) * 256;
  if (slab < 1) slab = 1;
  return slab;
}

// the same for the block-scaled half form of the intermediate (about half the bytes per row)
int64_t slab_rows_cap_z16(int64_t d) {
  int64_t slab = ((int64_t)128 << 20) / (z16_ld(d) * 2);
  if (slab >= 512) slab = (slab / 256) * 256;
  if (slab < 1) slab = 1;
  return slab;
}

// The plan's float32 intermediate for `stream`, at least `bytes` long (bytes <= cap = one full
// slab).  The first use on a stream allocates what the call needs, but at least 8 MB; a later
// call that needs more allocates the cap, once, and the outgrown buffer is kept until the plan is
// destroyed (queued launches and captured graphs still point at it).  So a stream sees at most
// two hipMalloc calls, nothing is freed and the stream is never waited for.  hipMalloc is not
// allowed while the stream is being captured: warm the plan up with the largest batch first.
// Per-call stream-ordered allocation was measured first: it added two stream operations to
// every call, 29 us per call on a 2-kernel program against 11 us of kernel time.
harp_status_t plan_scratch(const harp_plan_t *plan, hipStream_t stream, size_t bytes, size_t cap,
                           float **out) {
  std::lock_guard<std::mutex> lock(plan->scratch_mu);
  harp_plan::Scratch *slot = nullptr;
  for (auto &sc : plan->scratch)
    if (sc.stream == stream) slot = &sc;
  if (slot && slot->bytes >= bytes) {
    *out = slot->ptr;
    return HARP_OK;
  }
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &cs) != hipSuccess) {
    (void)hipGetLastError();
    return HARP_ERR_DEVICE;
  }
  if (cs != hipStreamCaptureStatusNone) return HARP_ERR_UNSUPPORTED;
  size_t want = slot ? cap : std::min(cap, std::max(bytes, (size_t)8 << 20));
  if (want < bytes) want = bytes;
  float *p = nullptr;
  if (hipMalloc((void **)&p, want) != hipSuccess) {
    (void)hipGetLastError();
    return HARP_ERR_OOM;
  }
  if (slot) {
    plan->retired.push_back(slot->ptr);
    slot->ptr = p;
    slot->bytes = want;
  } else {
    plan->scratch.push_back(harp_plan::Scratch{stream, p, want});
  }
  *out = p;
  return HARP_OK;
}

// Passes [p0, p1) of the program on row chunks, fused on chip.
harp_status_t run_chunk_passes(const harp_plan_t *plan, const HostProgram &hp, int p0, int p1,
                               const void *X, int64_t ldx, harp_dtype_t dt_in, void *Y, int64_t ldy,
                               harp_dtype_t dt_out, int64_t n, hipStream_t stream) {
  if (p1 - p0 == hp.n_chunk && dpp_supported(plan, hp.dpp, hp.chunk, X, ldx, dt_in, Y, ldy, dt_out))
    return launch_dpp_kernel(plan, hp.dpp, X, ldx, dt_in, Y, ldy, dt_out, n,
                             choose_pipe_rows(plan, n, plan->d / hp.chunk, hp.chunk), stream);
  if (pipe_supported(plan, hp.prog, p0, p1 - p0, hp.chunk, X, ldx, Y, ldy))
    return launch_pipe_kernel(plan, hp, p0, hp.chunk, X, ldx, dt_in, Y, ldy, dt_out, n,
                              choose_pipe_rows(plan, n, plan->d / hp.chunk, hp.chunk), stream);
  if (wave_supported(plan, hp.prog, p0, p1 - p0, hp.chunk, X, ldx, Y, ldy))
    return launch_wave_kernel(plan, hp, p0, p1 - p0, hp.chunk, X, ldx, dt_in, Y, ldy, dt_out, n,
                              stream);
  // tied parameters and in-kernel signs exist in the wave kernel only (16-byte aligned rows)
  if (plan->tied_K > 0) return HARP_ERR_UNSUPPORTED;
  if (radix_supported(plan, hp.prog, p0, p1 - p0, hp.chunk, X, ldx, Y, ldy))
    return launch_radix_kernel(plan, hp, p0, p1 - p0, hp.chunk, X, ldx, dt_in, Y, ldy, dt_out, n,
                               stream);
  return launch_tile_kernel(plan, hp.dev, p0, p1, hp.chunk, X, ldx, dt_in, Y, ldy, dt_out, n,
                            stream);
}

// The intermediate of a split program as block-scaled halves (2 bytes per coordinate instead of
// 4) for bf16 callers: one streamed dense stage of radix 3..8 next to the wave or the DPP
// kernel, for plans whose blocks are orthogonal (intermediate values then have the size of the
// row's own, and the format's 2^-12 per value is an eighth of the caller's own rounding).
bool split_uses_z16(const harp_plan_t *plan, const HostProgram &hp, const void *X, int64_t ldx,
                    harp_dtype_t dt_in, const void *Y, int64_t ldy, harp_dtype_t dt_out,
                    int64_t n = INT64_MAX) {
  if (!hp.z16 || dt_in != HARP_BF16 || dt_out != HARP_BF16) return false;
  // a few rows on chunks of 2048: launch latency counts, not bytes, and the float32 pair of
  // kernels measured 0.8 - 1.1 us less per launch inside a HIP graph (14336, n <= 32)
  if (n <= 32 && hp.chunk == 2048) return false;
  const int np = hp.prog.npass;
  const int nstream = np - hp.n_chunk;
  if (nstream < 1) return false;
  const int p0 = hp.chunk_first ? 0 : nstream, ps = hp.chunk_first ? hp.n_chunk : 0;
  const int64_t zl = z16_ld(plan->d);
  const void *cx = hp.chunk_first ? X : nullptr, *cy = hp.chunk_first ? nullptr : Y;
  const int64_t clx = hp.chunk_first ? ldx : zl, cly = hp.chunk_first ? zl : ldy;
  const harp_dtype_t zt = (harp_dtype_t)kDtZ16;
  // chunk kernels that read or write the format: the wave kernel and the DPP kernel
  if (!wave_supported(plan, hp.prog, p0, hp.n_chunk, hp.chunk, cx, clx, cy, cly) &&
      !dpp_supported(plan, hp.dpp, hp.chunk, cx, clx, hp.chunk_first ? dt_in : zt, cy, cly,
                     hp.chunk_first ? zt : dt_out))
    return false;
  // streamed stage: the small-radix kernel (the matrix-core kernel was measured with this
  // format and is not faster with it: it is bound by its LDS transposes, not by bytes)
  // (several streamed trips: the ones between two intermediates run in place on the halves)
  for (int k = 0; k < nstream; ++k) {
    const bool first = (k == 0), last = (k == nstream - 1);
    const bool from_caller = !hp.chunk_first && first, to_caller = hp.chunk_first && last;
    if (!stream_z16_supported(hp.prog.pass[ps + k], from_caller ? X : nullptr, from_caller ? ldx : zl,
                              to_caller ? Y : nullptr, to_caller ? ldy : zl))
      return false;
    // a trip with halves on both sides exists in the LDS-staged kernel only
    if (!from_caller && !to_caller &&
        (hp.prog.pass[ps + k].S % 256 != 0 || hp.prog.pass[ps + k].nq % 256 != 0))
      return false;
  }
  return true;
}

// Split program on rows [0, n): the chunk-local passes run fused on chip, every other pass is
// streamed through the float32 intermediate Z, which holds `slab` rows; rows are processed slab
// by slab so that Z stays small (it is written by one launch and read by the next: cache
// resident).
harp_status_t run_split(const harp_plan_t *plan, const HostProgram &hp, const void *X, int64_t ldx,
                        harp_dtype_t dt_in, void *Y, int64_t ldy, harp_dtype_t dt_out, int64_t n,
                        float *Z, int64_t slab, hipStream_t stream);

harp_status_t apply_dir(const harp_plan_t *plan, Direction dir, const void *X, int64_t ldx,
                        harp_dtype_t dt_in, void *Y, int64_t ldy, harp_dtype_t dt_out, int64_t n,
                        void *stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  const HostProgram *hpp = select_program(plan, dir, n, nullptr);
  if (!hpp) return HARP_ERR_UNSUPPORTED;
  const HostProgram &hp = *hpp;
  const int np = hp.prog.npass;
  if (hp.n_chunk == np)   // everything on chip, one launch
    return run_chunk_passes(plan, hp, 0, np, X, ldx, dt_in, Y, ldy, dt_out, n, stream);
  // transposed, one small dense stage above twelve radix-2 stages, bf16 rows: one launch, no
  // intermediate
  if (dpp_top_supported(plan, hp.dpp, X, ldx, dt_in, Y, ldy, dt_out))
    return launch_dpp_top_kernel(plan, hp.dpp, X, ldx, Y, ldy, n,
                                 choose_pipe_rows(plan, n, plan->d / hp.chunk, hp.chunk), stream);
  const int64_t d = plan->d;
  const bool z16 = split_uses_z16(plan, hp, X, ldx, dt_in, Y, ldy, dt_out, n);
  const int64_t slab_cap = z16 ? slab_rows_cap_z16(d) : slab_rows_cap(d);
  const int64_t slab = slab_cap > n ? n : slab_cap;
  const size_t row_bytes = z16 ? (size_t)z16_ld(d) * 2 : (size_t)d * 4;
  // one buffer per stream serves both forms: its full size is the larger of the two slabs
  const size_t cap = std::max((size_t)slab_rows_cap(d) * d * 4,
                              hp.z16 ? (size_t)slab_rows_cap_z16(d) * z16_ld(d) * 2 : (size_t)0);
  float *Z = nullptr;
  harp_status_t zst = plan_scratch(plan, stream, (size_t)slab * row_bytes, cap, &Z);
  if (zst != HARP_OK) return zst;
  return run_split(plan, hp, X, ldx, dt_in, Y, ldy, dt_out, n, Z, slab, stream);
}

harp_status_t run_split(const harp_plan_t *plan, const HostProgram &hp, const void *X, int64_t ldx,
                        harp_dtype_t dt_in, void *Y, int64_t ldy, harp_dtype_t dt_out, int64_t n,
                        float *Z, int64_t slab, hipStream_t stream) {
  const int64_t d = plan->d;
  const int np = hp.prog.npass;
  const int nstream = np - hp.n_chunk;
  const int nseg = nstream + 1;
  const bool allow_narrow = (dt_in == HARP_BF16 || dt_out == HARP_BF16);
  // bf16 on both sides, one streamed dense stage: the intermediate as block-scaled halves
  const bool z16 = split_uses_z16(plan, hp, X, ldx, dt_in, Y, ldy, dt_out, n);
  const harp_dtype_t z_dt = z16 ? (harp_dtype_t)kDtZ16 : HARP_F32;
  const int64_t z_ld = z16 ? z16_ld(d) : d;
  harp_status_t st = HARP_OK;
  for (int64_t r0 = 0; r0 < n && st == HARP_OK; r0 += slab) {
    const int64_t nr = (n - r0 < slab) ? n - r0 : slab;
    const void *src = (const char *)X + (size_t)r0 * ldx * esize(dt_in);
    int64_t src_ld = ldx;
    harp_dtype_t src_dt = dt_in;
    for (int seg = 0; seg < nseg && st == HARP_OK; ++seg) {
      const bool last = (seg == nseg - 1);
      void *dst = last ? (void *)((char *)Y + (size_t)r0 * ldy * esize(dt_out)) : (void *)Z;
      const int64_t dst_ld = last ? ldy : z_ld;
      const harp_dtype_t dst_dt = last ? dt_out : z_dt;
      const bool is_chunk = hp.chunk_first ? (seg == 0) : last;
      if (is_chunk) {
        const int p0 = hp.chunk_first ? 0 : nstream;
        st = run_chunk_passes(plan, hp, p0, p0 + hp.n_chunk, src, src_ld, src_dt, dst, dst_ld,
                              dst_dt, nr, stream);
      } else {
        const int p = hp.chunk_first ? hp.n_chunk + (seg - 1) : seg;
        st = launch_stream_pass(plan, hp, p, src, src_ld, src_dt, dst, dst_ld, dst_dt, nr,
                                allow_narrow, stream);
      }
      src = dst;
      src_ld = dst_ld;
      src_dt = dst_dt;
    }
  }
  return st;
}

harp_status_t rotate_impl(const harp_plan_t *pu, const harp_plan_t *pv, Direction dir,
                          const void *W, int64_t ldw, void *Wout, int64_t ldo, int64_t d_out,
                          int64_t d_in, harp_dtype_t dt, void *ws, size_t ws_bytes, void *stream) {
  if (dt != HARP_F32 && dt != HARP_BF16) return HARP_ERR_INVALID_ARG;
  if (d_out < 0 || d_in < 0) return HARP_ERR_INVALID_ARG;
  if (pu && pu->d != d_out) return HARP_ERR_INVALID_ARG;
  if (pv && pv->d != d_in) return HARP_ERR_INVALID_ARG;
  if (d_out == 0 || d_in == 0) return HARP_OK;
  if (!W || !Wout || ldw < d_in || ldo < d_in) return HARP_ERR_INVALID_ARG;
  size_t need = 0;
  harp_status_t st = harp_rotate_weight_workspace_size(pu, pv, d_out, d_in, dt, &need);
  if (st != HARP_OK) return st;
  if (need > 0 && (!ws || ws_bytes < need)) return HARP_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;

  if (!pu) {
    if (!pv) {
      if (W == Wout && ldw == ldo) return HARP_OK;
      return launch_copy2d(W, ldw, Wout, ldo, d_out, d_in, dt, s);
    }
    // rows of W through plan_V only
    return apply_dir(pv, dir, W, ldw, dt, Wout, ldo, dt, d_out, stream);
  }
  // Column side, radices up to 8: plan_U's stages run along the row index of the matrix in
  // place of a transposed copy (the same direction flag as the row side: U^T M uses the
  // forward stage order, U M the transposed one).  Intermediates stay in float32 so that a
  // bf16 matrix is rounded once, at the final store.
  const std::vector<ColPassHost> &cps = pu->colpass[dir];
  if (!cps.empty()) {
    float *A = (float *)ws;   // [d_out, d_in] float32, or block-scaled halves (see below)
    // plan_V as a split program with one streamed small-radix stage: that stage acts on the
    // columns and commutes with plan_U's stages, so it rides along with one column pass instead
    // of taking its own trip through device memory.  Forward: chunk passes of plan_V, then the
    // column passes; inverse: the column passes, then plan_V's chunk passes.
    const HostProgram *vhp = pv ? select_program(pv, dir, d_out, nullptr) : nullptr;
    // Workspace format.  A bf16 matrix between orthogonal processors travels through the
    // workspace as block-scaled halves (one power-of-two scale per 16 columns of a row, 2.06
    // bytes per entry instead of 4): each trip adds at most 2^-12 of an entry (or 2^-25 of its
    // segment's largest) where the caller's own element type rounds by 2^-9, and the matrix is
    // still rounded to bf16 once, at the last store.  It needs whole 128-column tiles in every
    // column pass and, on plan_V's side, the two-group DPP kernel, which reads and writes the
    // format (writing it going up, reading it going down); otherwise float32 as before.
    const harp_dtype_t ZT = (harp_dtype_t)kDtZ16;
    const int64_t zl = z16_ld(d_in);
    bool zws = dt == HARP_BF16 && pu->orthogonal && (!pv || pv->orthogonal) && !pu->f32_only &&
               !(pv && pv->f32_only) &&
               (cps.size() > 1 || pv) && (uintptr_t)ws % 16 == 0;
    for (size_t p = 0; p < cps.size() && zws; ++p)
      zws = col_z16_supported(cps[p].pass, W, ldw, Wout, ldo, d_out, d_in) &&
            col_z16_supported(cps[p].pass, A, zl, A, zl, d_out, d_in);
    // plan_V's on-chip passes with the halves on the workspace side
    auto chunk_z16_ok = [&]() {
      return dir == DIR_FWD ? dpp_supported(pv, vhp->dpp, vhp->chunk, W, ldw, HARP_BF16, A, zl, ZT)
                            : dpp_supported(pv, vhp->dpp, vhp->chunk, A, zl, ZT, Wout, ldo, HARP_BF16);
    };
    if (zws && pv && (!vhp || !chunk_z16_ok())) zws = false;
    int fuse = -1;
    const PassDesc *vp = nullptr;
    const bool one_streamed = vhp && vhp->n_chunk + 1 == vhp->prog.npass;
    auto find_fuse = [&](bool z) {
      const harp_dtype_t wt = z ? ZT : HARP_F32;
      const int64_t wld = z ? zl : d_in;
      for (int p = (int)cps.size() - 1; p >= 0; --p) {
        const bool first = (p == 0), last = (p + 1 == (int)cps.size());
        // what this pass reads and writes in the fused order
        const bool reads_w = (dir == DIR_TRN) && first;
        const bool writes_out = (dir == DIR_FWD) && last;
        const void *src = reads_w ? W : (const void *)A;
        const void *dst = writes_out ? (const void *)Wout : (const void *)A;
        if (colrow_supported(pu, cps[p].pass, *vp, src, reads_w ? ldw : wld, reads_w ? dt : wt, dst,
                             writes_out ? ldo : wld, writes_out ? dt : wt, d_out, d_in))
          return p;
      }
      return -1;
    };
    // (the streamed stage on its own trip between halves and the caller's matrix)
    bool own_trip = false;
    if (one_streamed) {
      vp = &vhp->prog.pass[vhp->chunk_first ? vhp->n_chunk : 0];
      if (zws) {
        const bool fwd = (dir == DIR_FWD);
        fuse = find_fuse(true);
        own_trip = stream_z16_supported(*vp, fwd ? (const void *)A : W, fwd ? zl : ldw,
                                        fwd ? Wout : (void *)A, fwd ? ldo : zl);
        if (fuse < 0 && !own_trip) zws = false;
      }
      if (fuse < 0 && !zws) fuse = find_fuse(false);
    } else if (zws && pv && vhp->n_chunk != vhp->prog.npass) {
      zws = false;   // several streamed trips: plan_V runs on its own, through float32
    }
    if (zws && pv && fuse < 0 && !own_trip && vhp->n_chunk != vhp->prog.npass) zws = false;
    const harp_dtype_t wt = zws ? ZT : HARP_F32;
    const int64_t wld = zws ? zl : d_in;
    const void *src = W;
    int64_t src_ld = ldw;
    harp_dtype_t src_dt = dt;
    // Halves in the workspace and every column pass on the register-tile kernel: plan_V's streamed
    // stage then takes its own trip (its kernel runs at the copy rate on 2-byte entries) instead
    // of riding along with a column pass on the LDS-tile kernel: at 8192 x 28672 the forward map
    // measured 0.90 against 0.93 ms, the inverse the same either way.  Forward: chunks, column
    // passes, streamed stage; inverse: streamed stage, column passes, chunks.
    // (also when no column pass can take the stage along: a radix-2 stage on the top digit)
    if (zws && own_trip) {
      bool regs = true;
      for (size_t p = 0; p < cps.size(); ++p) regs = regs && col_pass_in_registers(cps[p].pass, d_in);
      const int ps = vhp->chunk_first ? vhp->n_chunk : 0, c0 = vhp->chunk_first ? 0 : 1;
      const bool fwd = (dir == DIR_FWD);
      if (regs || fuse < 0) {
        if (fwd)
          st = run_chunk_passes(pv, *vhp, c0, c0 + vhp->n_chunk, W, ldw, dt, A, zl, ZT, d_out, s);
        else
          st = launch_stream_pass(pv, *vhp, ps, W, ldw, dt, A, zl, ZT, d_out, true, s);
        for (size_t p = 0; p < cps.size() && st == HARP_OK; ++p)
          st = launch_col_pass(pu, cps[p].dev, cps[p].pass, A, zl, ZT, A, zl, ZT, d_out, d_in, s);
        if (st != HARP_OK) return st;
        if (fwd) return launch_stream_pass(pv, *vhp, ps, A, zl, ZT, Wout, ldo, dt, d_out, true, s);
        return run_chunk_passes(pv, *vhp, c0, c0 + vhp->n_chunk, A, zl, ZT, Wout, ldo, dt, d_out, s);
      }
    }
    if (fuse >= 0) {
      const int c0 = vhp->chunk_first ? 0 : 1;
      if (dir == DIR_FWD) {
        st = run_chunk_passes(pv, *vhp, c0, c0 + vhp->n_chunk, W, ldw, dt, A, wld, wt, d_out, s);
        if (st != HARP_OK) return st;
        src = A;
        src_ld = wld;
        src_dt = wt;
      }
      for (size_t p = 0; p < cps.size(); ++p) {
        const bool to_out = (dir == DIR_FWD) && (p + 1 == cps.size());
        void *dst = to_out ? Wout : (void *)A;
        const int64_t dst_ld = to_out ? ldo : wld;
        const harp_dtype_t dst_dt = to_out ? dt : wt;
        if ((int)p == fuse)
          st = launch_colrow_pass(pu, cps[p].dev, cps[p].pass, *vp, src, src_ld, src_dt, dst, dst_ld,
                                  dst_dt, d_out, d_in, s);
        else
          st = launch_col_pass(pu, cps[p].dev, cps[p].pass, src, src_ld, src_dt, dst, dst_ld, dst_dt,
                               d_out, d_in, s);
        if (st != HARP_OK) return st;
        src = dst;
        src_ld = dst_ld;
        src_dt = dst_dt;
      }
      if (dir == DIR_TRN)
        st = run_chunk_passes(pv, *vhp, c0, c0 + vhp->n_chunk, A, wld, wt, Wout, ldo, dt, d_out, s);
      return st;
    }
    // plan_V on its own: before the column passes, or (halves, inverse map: the DPP kernel reads
    // the format only going down) behind them -- the two sides commute
    const bool v_last = zws && pv && dir == DIR_TRN;
    if (pv && !v_last) {
      if (zws)
        st = run_chunk_passes(pv, *vhp, 0, vhp->prog.npass, W, ldw, dt, A, wld, wt, d_out, s);
      else
        st = apply_dir(pv, dir, W, ldw, dt, A, d_in, HARP_F32, d_out, stream);
      if (st != HARP_OK) return st;
      src = A;
      src_ld = wld;
      src_dt = wt;
    }
    for (size_t p = 0; p < cps.size(); ++p) {
      const bool last = (p + 1 == cps.size()) && !v_last;
      void *dst = last ? Wout : (void *)A;
      const int64_t dst_ld = last ? ldo : wld;
      const harp_dtype_t dst_dt = last ? dt : wt;
      st = launch_col_pass(pu, cps[p].dev, cps[p].pass, src, src_ld, src_dt, dst, dst_ld, dst_dt,
                           d_out, d_in, s);
      if (st != HARP_OK) return st;
      src = dst;
      src_ld = dst_ld;
      src_dt = dst_dt;
    }
    if (v_last)
      st = run_chunk_passes(pv, *vhp, 0, vhp->prog.npass, A, wld, wt, Wout, ldo, dt, d_out, s);
    return st;
  }
  // Otherwise: (U^T M)^T = M^T U, i.e. the rows of M^T go through plan_U as a row processor.
  const size_t mat = (size_t)d_out * d_in * 4;
  float *A = (float *)ws;                                   // [d_out, d_in] (only with plan_V)
  float *B = pv ? (float *)((char *)ws + mat) : (float *)ws;  // [d_in, d_out]
  if (pv) {
    st = apply_dir(pv, dir, W, ldw, dt, A, d_in, HARP_F32, d_out, stream);
    if (st != HARP_OK) return st;
    st = launch_transpose(A, d_in, HARP_F32, B, d_out, HARP_F32, d_out, d_in, s);
  } else {
    st = launch_transpose(W, ldw, dt, B, d_out, HARP_F32, d_out, d_in, s);
  }
  if (st != HARP_OK) return st;
  st = apply_dir(pu, dir, B, d_out, HARP_F32, B, d_out, HARP_F32, d_in, stream);
  if (st != HARP_OK) return st;
  return launch_transpose(B, d_out, HARP_F32, Wout, ldo, dt, d_in, d_out, s);
}

}  // namespace

namespace harp {

// Rows per tile of the pipelined kernel: a workgroup handles R rows of one chunk, so a launch
// has nchunk * ceil(n / R) workgroups.  Aim at one workgroup slot per compute unit (two for
// the 2048-coordinate kernel, whose workgroups are half as large) with tiles of <= 32 rows,
// otherwise several waves of nearly equal tiles.
int choose_pipe_rows(const harp_plan *plan, int64_t n, int64_t nchunk, int chunk) {
  if (plan->rows_override > 0) return plan->rows_override;
  const int64_t slots =
      (int64_t)(plan->num_cu > 0 ? plan->num_cu : 256) * (chunk <= 1024 ? 4 : (chunk <= 2048 ? 2 : 1));
  const int64_t waves = (n * nchunk + slots * 32 - 1) / (slots * 32);
  int64_t per_chunk = (slots * waves) / nchunk;   // workgroups available to one chunk index
  if (per_chunk < 1) per_chunk = 1;
  int64_t R = (n + per_chunk - 1) / per_chunk;
  if (R < 1) R = 1;
  if (R > 1 && (R & 1)) ++R;   // the kernel moves rows in pairs
  return (int)R;
}

const HostProgram *select_program(const harp_plan *plan, Direction dir, int64_t n,
                                  const char **name) {
  int algo = plan->algo;
  if (algo == HARP_ALGO_AUTO) {
    // rows longer than one on-chip chunk: split at every batch size (measured down to one row:
    // two short launches beat one workgroup per row re-reading the whole parameter image)
    const HostProgram &sp = plan->prog[HARP_ALGO_SPLIT][dir];
    if (sp.ok && (!sp.optional || (dir == DIR_FWD && n >= 512)))
      algo = HARP_ALGO_SPLIT;
    else
      algo = plan->prog[HARP_ALGO_FUSED][dir].ok ? HARP_ALGO_FUSED : HARP_ALGO_GENERIC;
  }
  const HostProgram &hp = plan->prog[algo][dir];
  if (!hp.ok) return nullptr;
  if (name)
    *name = (algo == HARP_ALGO_SPLIT) ? "split_chunk_stream"
                                      : (algo == HARP_ALGO_FUSED ? "tile_fused" : "tile_generic");
  return &hp;
}

}  // namespace harp

// Int8 images for the run-time reconstruction (HARP_THETA_IN_KERNEL).  A stage qualifies when
// its radix is 4 or 8 and its mixer the Hadamard matrix or the identity; its image is attached
// to every PASS_SMALL pass of that stage in every program, and the chain kernel of harp_radix.hip
// takes the reconstructing variant when all passes of its chunk carry one.
harp_status_t harp::plan_attach_theta_int8(harp_plan *plan, const int8_t *const *codes,
                                           const float *const *scales,
                                           const int32_t *mixer_kinds, const int8_t *signs) {
  if (!plan || !codes || !scales) return HARP_ERR_INVALID_ARG;
  if (plan->tied_K > 0) return HARP_OK;
  const int m = plan->m;
  const int64_t d = plan->d;
  bool any = false;
  for (int t = 0; t < m; ++t) {
    const int b = plan->radices[t];
    const int kind = mixer_kinds ? mixer_kinds[t] : HARP_MIXER_HADAMARD;
    if ((b != 4 && b != 8) || (kind != HARP_MIXER_HADAMARD && kind != HARP_MIXER_IDENTITY)) continue;
    const int64_t nq = d / b;
    const int npar = b * (b - 1) / 2;
    const int rec = (b == 8) ? 32 : 8;           // bytes per block
    const int pieces = (b == 8) ? 2 : 1, psz = rec / pieces;
    std::vector<uint8_t> img((size_t)nq * rec + (size_t)nq * 4, 0);
    const bool with_signs = signs && plan->strides[t] == 1;   // stage 0
    for (int64_t c = 0; c < nq; ++c) {
      uint8_t r[32] = {0};
      for (int i = 0; i < npar; ++i) r[i] = (uint8_t)codes[t][(size_t)c * npar + i];
      if (with_signs)
        for (int j = 0; j < b; ++j)
          if (signs[c * b + j] < 0) r[npar] |= (uint8_t)(1u << j);
      for (int k = 0; k < pieces; ++k)
        memcpy(img.data() + ((size_t)k * nq + c) * psz, r + k * psz, psz);
      memcpy(img.data() + (size_t)nq * rec + (size_t)c * 4, &scales[t][c], 4);
    }
    void *dimg = nullptr;
    if (hipMalloc(&dimg, img.size()) != hipSuccess) return HARP_ERR_OOM;
    plan->dev_allocs.push_back(dimg);
    if (hipMemcpy(dimg, img.data(), img.size(), hipMemcpyHostToDevice) != hipSuccess)
      return HARP_ERR_DEVICE;
    const int32_t fl = (kind == HARP_MIXER_HADAMARD ? 1 : 0) | (with_signs ? 2 : 0);
    for (int algo = HARP_ALGO_GENERIC; algo <= HARP_ALGO_SPLIT; ++algo)
      for (int dir = 0; dir < 2; ++dir) {
        HostProgram &hp = plan->prog[algo][dir];
        if (!hp.ok) continue;
        // A radix-2 pass in the two-shear or lifting form leaves scales or signs pending on its
        // coordinates, which the plan builder folds into the rows of the next dense block: a
        // block behind such a pass is not the one the codes describe.
        bool clean = true;
        for (int p = 0; p < hp.prog.npass; ++p) {
          PassDesc &pd = hp.prog.pass[p];
          if (pd.kind == PASS_POW2_LIFT || pd.kind == PASS_POW2_LIFT_LD ||
              pd.kind == PASS_POW2_SCALED || pd.kind == PASS_POW2_SCALED_LD)
            clean = false;
          if (!clean) continue;
          if (pd.kind != PASS_SMALL || pd.b != b || pd.S != plan->strides[t] || pd.tied) continue;
          pd.q8 = dimg;
          pd.q8_flags = fl;
          any = true;
        }
      }
  }
  if (!any) return HARP_OK;
  for (int algo = HARP_ALGO_GENERIC; algo <= HARP_ALGO_SPLIT; ++algo)
    for (int dir = 0; dir < 2; ++dir) {
      HostProgram &hp = plan->prog[algo][dir];
      if (!hp.ok || !hp.dev) continue;
      if (hipMemcpy(const_cast<Program *>(hp.dev), &hp.prog, sizeof(Program),
                    hipMemcpyHostToDevice) != hipSuccess)
        return HARP_ERR_DEVICE;
    }
  plan->theta_in_kernel = true;
  return HARP_OK;
}

harp_status_t harp::plan_create_impl(harp_plan **out, int64_t d, int32_t m, const int32_t *radices,
                                     const float *const *blocks, const int8_t *signs,
                                     uint32_t flags, int32_t tied_K) {
  if (!out || !radices || !blocks) return HARP_ERR_INVALID_ARG;
  if (flags & ~(uint32_t)(HARP_VALIDATE_ORTHO | HARP_BLOCKS_ON_DEVICE | HARP_F32_INTERMEDIATES))
    return HARP_ERR_INVALID_ARG;
  if (d < 2) return HARP_ERR_INVALID_ARG;
  if (m < 1 || m > HARP_MAX_STAGES) return HARP_ERR_BAD_SCHEDULE;
  int64_t prod = 1;
  for (int t = 0; t < m; ++t) {
    if (radices[t] < 2) return HARP_ERR_BAD_SCHEDULE;
    if (prod > d) return HARP_ERR_BAD_SCHEDULE;
    prod *= radices[t];
  }
  if (prod != d) return HARP_ERR_BAD_SCHEDULE;
  for (int t = 0; t < m; ++t)
    if (!blocks[t]) return HARP_ERR_INVALID_ARG;
  for (int t = 0; t < m; ++t)
    if (radices[t] > HARP_MAX_RADIX) return HARP_ERR_UNSUPPORTED;
  if (d > (int64_t)1 << 24) return HARP_ERR_UNSUPPORTED;

  harp_plan *plan = new (std::nothrow) harp_plan();
  if (!plan) return HARP_ERR_OOM;
  harp_status_t st = HARP_OK;
  std::vector<std::vector<float>> host_copy;
  std::vector<int8_t> host_signs;
  std::vector<const float *> blk(m);
  try {
    plan->d = d;
    plan->m = m;
    if (tied_K > 0) {
      plan->tied_K = tied_K;
      plan->tied_n2 = d / tied_K;
    }
    {
      const char *e = getenv("HARP_NO_MFMA");   // read once, here: launches never look at the environment
      plan->no_mfma = e && *e && atoi(e) != 0;
    }
    plan->radices.assign(radices, radices + m);
    plan->strides.resize(m);
    int64_t s = 1;
    for (int t = 0; t < m; ++t) {
      plan->strides[t] = s;
      s *= radices[t];
    }
    if (flags & HARP_BLOCKS_ON_DEVICE) {
      host_copy.resize(m);
      for (int t = 0; t < m && st == HARP_OK; ++t) {
        host_copy[t].resize((size_t)d * radices[t]);
        if (hipMemcpy(host_copy[t].data(), blocks[t], (size_t)d * radices[t] * 4,
                      hipMemcpyDeviceToHost) != hipSuccess)
          st = HARP_ERR_DEVICE;
        blk[t] = host_copy[t].data();
      }
      if (st == HARP_OK && signs) {
        host_signs.resize(d);
        if (hipMemcpy(host_signs.data(), signs, (size_t)d, hipMemcpyDeviceToHost) != hipSuccess)
          st = HARP_ERR_DEVICE;
        signs = host_signs.data();
      }
    } else {
      for (int t = 0; t < m; ++t) blk[t] = blocks[t];
    }
    if (st == HARP_OK && signs)
      for (int64_t i = 0; i < d; ++i)
        if (signs[i] != 1 && signs[i] != -1) {
          st = HARP_ERR_INVALID_ARG;
          break;
        }
    // every block entry must be finite; optionally orthogonal
    for (int t = 0; t < m && st == HARP_OK; ++t) {
      const int b = radices[t];
      const int64_t D = d / b;
      const float *K = blk[t];
      for (int64_t i = 0; i < D * b * b; ++i)
        if (!std::isfinite(K[i])) {
          st = HARP_ERR_INVALID_ARG;
          break;
        }
      // orthogonality of every block (always recorded: kernels that rely on intermediate values
      // having the size of the row's own ask for it; an error only with HARP_VALIDATE_ORTHO)
      bool ortho = true;
      if (st == HARP_OK) {
        for (int64_t c = 0; c < D && ortho; ++c) {
          const float *k = K + c * b * b;
          for (int i = 0; i < b && ortho; ++i)
            for (int j = i; j < b; ++j) {
              double acc = 0.0;
              for (int r = 0; r < b; ++r) acc += (double)k[r * b + i] * (double)k[r * b + j];
              if (std::fabs(acc - (i == j ? 1.0 : 0.0)) > 1e-5) {
                ortho = false;
                break;
              }
            }
        }
      }
      if (!ortho) {
        plan->orthogonal = false;
        if (flags & HARP_VALIDATE_ORTHO) st = HARP_ERR_NOT_ORTHOGONAL;
      }
    }
    plan->f32_only = (flags & HARP_F32_INTERMEDIATES) != 0;
    // ---- device side -------------------------------------------------------------
    if (st == HARP_OK) {
      int dev = 0;
      hipDeviceProp_t prop;
      if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        st = HARP_ERR_DEVICE;
      } else {
        plan->device = dev;
        plan->num_cu = prop.multiProcessorCount;
        int lds = 0;
        if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) !=
            hipSuccess)
          lds = (int)prop.sharedMemPerBlock;
        plan->lds_bytes = lds;
      }
    }
    for (int algo = HARP_ALGO_GENERIC; algo <= HARP_ALGO_SPLIT && st == HARP_OK; ++algo)
      for (int dir = 0; dir < 2 && st == HARP_OK; ++dir) {
        HostProgram &hp = plan->prog[algo][dir];
        std::vector<float> image;
        std::vector<size_t> offsets;
        std::vector<std::vector<uint16_t>> aux;
        if (!build_program(plan, blk, signs, algo, (Direction)dir, hp, image, offsets, aux)) {
          hp.ok = false;
          continue;
        }
        // whole-row programs need one float32 row in LDS
        if (algo != HARP_ALGO_SPLIT && (int64_t)d * 4 > plan->lds_bytes) {
          hp.ok = false;
          continue;
        }
        float *dimg = nullptr;
        if (hipMalloc((void **)&dimg, image.size() * 4) != hipSuccess) {
          st = HARP_ERR_OOM;
          break;
        }
        plan->dev_allocs.push_back(dimg);
        if (hipMemcpy(dimg, image.data(), image.size() * 4, hipMemcpyHostToDevice) != hipSuccess) {
          st = HARP_ERR_DEVICE;
          break;
        }
        if (hp.dpp.host_off >= 0) hp.dpp.img = dimg + hp.dpp.host_off;
        for (int p = 0; p < hp.prog.npass; ++p) {
          hp.prog.pass[p].params = dimg + offsets[p];
          hp.prog.pass[p].aux = nullptr;
          if (!aux[p].empty() && st == HARP_OK) {
            void *da = nullptr;
            if (hipMalloc(&da, aux[p].size() * 2) != hipSuccess) {
              st = HARP_ERR_OOM;
              break;
            }
            plan->dev_allocs.push_back(da);
            if (hipMemcpy(da, aux[p].data(), aux[p].size() * 2, hipMemcpyHostToDevice) !=
                hipSuccess) {
              st = HARP_ERR_DEVICE;
              break;
            }
            hp.prog.pass[p].aux = da;
          }
        }
        if (st != HARP_OK) break;
        Program *dprog = nullptr;
        if (hipMalloc((void **)&dprog, sizeof(Program)) != hipSuccess) {
          st = HARP_ERR_OOM;
          break;
        }
        plan->dev_allocs.push_back(dprog);
        if (hipMemcpy(dprog, &hp.prog, sizeof(Program), hipMemcpyHostToDevice) != hipSuccess) {
          st = HARP_ERR_DEVICE;
          break;
        }
        hp.dev = dprog;
      }
    if (st == HARP_OK && !plan->prog[HARP_ALGO_GENERIC][0].ok && !plan->prog[HARP_ALGO_SPLIT][0].ok)
      st = HARP_ERR_UNSUPPORTED;
    if (st == HARP_OK && tied_K > 0) {
      // both directions as wave kernel on the slices + matrix-core kernel for the table
      bool ok = !plan->no_mfma;
      for (int dir = 0; dir < 2 && ok; ++dir) {
        const HostProgram &hp = plan->prog[HARP_ALGO_SPLIT][dir];
        ok = hp.ok && hp.n_chunk + 1 == hp.prog.npass;
        if (!ok) break;
        const int p0 = hp.chunk_first ? 0 : 1, ps = hp.chunk_first ? hp.n_chunk : 0;
        ok = wave_supported(plan, hp.prog, p0, hp.n_chunk, hp.chunk, nullptr, 8, nullptr, 8) &&
             mfma_pass_supported(hp.prog.pass[ps], nullptr, 8, nullptr, 8);
      }
      if (!ok) st = HARP_ERR_UNSUPPORTED;
    }
    if (st == HARP_OK && signs) {
      int8_t *ds = nullptr;
      if (hipMalloc((void **)&ds, (size_t)d) != hipSuccess) {
        st = HARP_ERR_OOM;
      } else {
        plan->dev_allocs.push_back(ds);
        if (hipMemcpy(ds, signs, (size_t)d, hipMemcpyHostToDevice) != hipSuccess) st = HARP_ERR_DEVICE;
        plan->dev_signs = ds;
      }
    }
    // Column-mode image (the plan as the U side of a weight rotation, and the blocks the
    // gradient kernels read): per direction the dense effective blocks [d / b][b][b] of every
    // stage in execution order, and -- when every radix is at most 8 -- the passes over them.
    bool col_ok = true;
    for (int t = 0; t < m; ++t) col_ok = col_ok && radices[t] <= 8;
    // (a plan with tied parameters keeps no expanded per-stage images: it cannot be the U side of
    // a column-mode rotation and has no block gradients)
    for (int dir = 0; dir < 2 && st == HARP_OK && tied_K == 0; ++dir) {
      std::vector<StageEff> eff;
      build_effective(plan, blk, signs, HARP_ALGO_GENERIC, (Direction)dir, false, eff);
      size_t total = 0;
      for (const StageEff &se : eff) total += se.dense.size();
      std::vector<float> image(total);
      float *dimg = nullptr;
      if (hipMalloc((void **)&dimg, total * 4) != hipSuccess) {
        st = HARP_ERR_OOM;
        break;
      }
      plan->dev_allocs.push_back(dimg);
      size_t off = 0;
      for (const StageEff &se : eff) {
        std::copy(se.dense.begin(), se.dense.end(), image.begin() + off);
        plan->col[dir].push_back(ColStage{se.b, (int32_t)se.s, dimg + off});
        off += se.dense.size();
      }
      if (hipMemcpy(dimg, image.data(), total * 4, hipMemcpyHostToDevice) != hipSuccess) {
        st = HARP_ERR_DEVICE;
        break;
      }
      // Gradient path: a stage of radix 9..64 (and its transpose, for the gradient passed back)
      // runs on the matrix cores like the streamed stage of a split program, from the same
      // dense blocks as the vector kernels (float32 operand tiles; the image also carries the
      // bf16 tiles the kernel's other variant reads).
      if (dir == DIR_FWD) {
        plan->grad_mfma[0].assign(eff.size(), PassDesc{});
        plan->grad_mfma[1].assign(eff.size(), PassDesc{});
        for (size_t t = 0; t < eff.size() && st == HARP_OK; ++t) {
          const StageEff &se = eff[t];
          const int b = se.b;
          if (b < 9 || b > HARP_MAX_RADIX || se.s % 16 != 0) continue;
          const int64_t nq = d / b;
          const int KT = (b + 15) / 16;
          const size_t per = (size_t)KT * KT * 2 * 64 * 4, per32 = (size_t)KT * KT * 64 * 4;
          std::vector<uint16_t> a(per * nq + 2 * per32 * nq);
          std::vector<float> kt((size_t)b * b);
          for (int tr = 0; tr < 2 && st == HARP_OK; ++tr) {
            float *a32 = reinterpret_cast<float *>(a.data() + per * nq);
            for (int64_t q = 0; q < nq; ++q) {
              const float *K = se.dense.data() + (size_t)q * b * b;
              if (tr)
                for (int r = 0; r < b; ++r)
                  for (int r2 = 0; r2 < b; ++r2) kt[(size_t)r * b + r2] = K[(size_t)r2 * b + r];
              pack_mfma_block(tr ? kt.data() : K, b, a.data() + per * q, a32 + per32 * q);
            }
            void *da = nullptr;
            if (hipMalloc(&da, a.size() * 2) != hipSuccess) {
              st = HARP_ERR_OOM;
              break;
            }
            plan->dev_allocs.push_back(da);
            if (hipMemcpy(da, a.data(), a.size() * 2, hipMemcpyHostToDevice) != hipSuccess) {
              st = HARP_ERR_DEVICE;
              break;
            }
            PassDesc pd{};
            pd.kind = PASS_GENERIC;
            pd.b = b;
            pd.k = 1;
            pd.P = b;
            pd.S = (int32_t)se.s;
            pd.nq = (int32_t)nq;
            pd.nqp = (int32_t)nq;
            pd.V = b * b;
            pd.aux = da;
            plan->grad_mfma[tr][t] = pd;
          }
        }
        if (st != HARP_OK) break;
      }
      if (!col_ok || !build_col_passes(plan, (Direction)dir, plan->colpass[dir])) {
        plan->colpass[dir].clear();
        continue;
      }
      ColPass *dp = nullptr;
      const size_t np = plan->colpass[dir].size();
      if (hipMalloc((void **)&dp, np * sizeof(ColPass)) != hipSuccess) {
        st = HARP_ERR_OOM;
        break;
      }
      plan->dev_allocs.push_back(dp);
      for (size_t i = 0; i < np && st == HARP_OK; ++i) {
        ColPassHost &ph = plan->colpass[dir][i];
        uint32_t *dtab = nullptr;
        if (hipMalloc((void **)&dtab, ph.ptab.size() * 4) != hipSuccess) {
          st = HARP_ERR_OOM;
          break;
        }
        plan->dev_allocs.push_back(dtab);
        if (hipMemcpy(dtab, ph.ptab.data(), ph.ptab.size() * 4, hipMemcpyHostToDevice) !=
            hipSuccess) {
          st = HARP_ERR_DEVICE;
          break;
        }
        ph.pass.ptab = dtab;
        if (hipMemcpy(dp + i, &plan->colpass[dir][i].pass, sizeof(ColPass),
                      hipMemcpyHostToDevice) != hipSuccess)
          st = HARP_ERR_DEVICE;
        plan->colpass[dir][i].dev = dp + i;
      }
    }
  } catch (const std::bad_alloc &) {
    st = HARP_ERR_OOM;
  }
  if (st != HARP_OK) {
    harp_plan_destroy(plan);
    return st;
  }
  *out = plan;
  return HARP_OK;
}

extern "C" {

harp_status_t harp_plan_create(harp_plan_t **out, int64_t d, int32_t m, const int32_t *radices,
                               const float *const *blocks, const int8_t *signs, uint32_t flags) {
  return plan_create_impl(out, d, m, radices, blocks, signs, flags, 0);
}

harp_status_t harp_plan_destroy(harp_plan_t *plan) {
  if (!plan) return HARP_OK;
  harp_status_t st = HARP_OK;
  for (void *p : plan->dev_allocs)
    if (p && hipFree(p) != hipSuccess) st = HARP_ERR_DEVICE;
  for (auto &sc : plan->scratch)
    if (sc.ptr && hipFree(sc.ptr) != hipSuccess) st = HARP_ERR_DEVICE;
  for (void *p : plan->retired)
    if (p && hipFree(p) != hipSuccess) st = HARP_ERR_DEVICE;
  delete plan;
  return st;
}

harp_status_t harp_apply(const harp_plan_t *plan, const void *X, int64_t ldx, void *Y, int64_t ldy,
                         int64_t n, harp_dtype_t dt, void *stream) {
  harp_status_t st = check_apply_args(plan, X, ldx, Y, ldy, n, dt);
  if (st != HARP_OK || n == 0) return st;
  return apply_dir(plan, DIR_FWD, X, ldx, dt, Y, ldy, dt, n, stream);
}

harp_status_t harp_apply_transpose(const harp_plan_t *plan, const void *X, int64_t ldx, void *Y,
                                   int64_t ldy, int64_t n, harp_dtype_t dt, void *stream) {
  harp_status_t st = check_apply_args(plan, X, ldx, Y, ldy, n, dt);
  if (st != HARP_OK || n == 0) return st;
  return apply_dir(plan, DIR_TRN, X, ldx, dt, Y, ldy, dt, n, stream);
}

harp_status_t harp_apply_noalloc(const harp_plan_t *plan, const void *X, int64_t ldx, void *Y,
                                 int64_t ldy, int64_t n, harp_dtype_t dt, int32_t transpose,
                                 void *stream) {
  harp_status_t st = check_apply_args(plan, X, ldx, Y, ldy, n, dt);
  if (st != HARP_OK || n == 0) return st;
  if (transpose != 0 && transpose != 1) return HARP_ERR_INVALID_ARG;
  const Direction dir = transpose ? DIR_TRN : DIR_FWD;
  const HostProgram *hpp = select_program(plan, dir, n, nullptr);
  if (!hpp) return HARP_ERR_UNSUPPORTED;
  const HostProgram &hp = *hpp;
  if (hp.n_chunk == hp.prog.npass)   // one launch, no intermediate at all
    return run_chunk_passes(plan, hp, 0, hp.prog.npass, X, ldx, dt, Y, ldy, dt, n, (hipStream_t)stream);
  if (dpp_top_supported(plan, hp.dpp, X, ldx, dt, Y, ldy, dt))   // one launch, no intermediate
    return launch_dpp_top_kernel(plan, hp.dpp, X, ldx, Y, ldy, n,
                                 choose_pipe_rows(plan, n, plan->d / hp.chunk, hp.chunk),
                                 (hipStream_t)stream);
  // the whole batch has to fit the library's own array: no slab loop, a clear refusal instead
  if ((size_t)n > HARP_NOALLOC_SCRATCH_BYTES / ((size_t)plan->d * 4)) return HARP_ERR_UNSUPPORTED;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return HARP_ERR_DEVICE;
  }
  if (dev != plan->device) return HARP_ERR_INVALID_ARG;   // the plan's images live on its own device
  float *Z = nullptr;
  st = noalloc_scratch(dev, &Z);
  if (st != HARP_OK) return st;
  return run_split(plan, hp, X, ldx, dt, Y, ldy, dt, n, Z, n, (hipStream_t)stream);
}

int64_t harp_apply_noalloc_max_rows(const harp_plan_t *plan) {
  if (!plan) return -1;
  const HostProgram *hpp = select_program(plan, DIR_FWD, 1, nullptr);
  const HostProgram *hpt = select_program(plan, DIR_TRN, 1, nullptr);
  if (!hpp || !hpt) return -1;
  const bool split = hpp->n_chunk != hpp->prog.npass || hpt->n_chunk != hpt->prog.npass ||
                     plan->prog[HARP_ALGO_SPLIT][DIR_FWD].ok;
  if (!split) return INT64_MAX;
  return (int64_t)(HARP_NOALLOC_SCRATCH_BYTES / ((size_t)plan->d * 4));
}

harp_status_t harp_rotate_weight_workspace_size(const harp_plan_t *plan_U,
                                                const harp_plan_t *plan_V, int64_t d_out,
                                                int64_t d_in, harp_dtype_t dt, size_t *bytes) {
  if (!bytes) return HARP_ERR_INVALID_ARG;
  if (dt != HARP_F32 && dt != HARP_BF16) return HARP_ERR_INVALID_ARG;
  if (d_out < 0 || d_in < 0) return HARP_ERR_INVALID_ARG;
  if (plan_U && plan_U->d != d_out) return HARP_ERR_INVALID_ARG;
  if (plan_V && plan_V->d != d_in) return HARP_ERR_INVALID_ARG;
  // One float32 copy of the matrix when plan_U runs as column passes along the row index (every
  // radix <= 8); the transposing path (a radix above 8 in plan_U) needs a second one for the
  // transposed copy when plan_V is given too.
  const size_t mat = (size_t)d_out * (size_t)d_in * 4;
  const bool col_path = plan_U && !plan_U->colpass[0].empty() && !plan_U->colpass[1].empty();
  *bytes = !plan_U ? 0 : ((plan_V && !col_path) ? 2 * mat : mat);
  return HARP_OK;
}

harp_status_t harp_rotate_weight(const harp_plan_t *plan_U, const harp_plan_t *plan_V,
                                 const void *W, int64_t ldw, void *Wout, int64_t ldo,
                                 int64_t d_out, int64_t d_in, harp_dtype_t dt, void *workspace,
                                 size_t workspace_bytes, void *stream) {
  return rotate_impl(plan_U, plan_V, DIR_FWD, W, ldw, Wout, ldo, d_out, d_in, dt, workspace,
                     workspace_bytes, stream);
}

harp_status_t harp_rotate_weight_inverse(const harp_plan_t *plan_U, const harp_plan_t *plan_V,
                                         const void *W, int64_t ldw, void *Wout, int64_t ldo,
                                         int64_t d_out, int64_t d_in, harp_dtype_t dt,
                                         void *workspace, size_t workspace_bytes, void *stream) {
  return rotate_impl(plan_U, plan_V, DIR_TRN, W, ldw, Wout, ldo, d_out, d_in, dt, workspace,
                     workspace_bytes, stream);
}

harp_status_t harp_grad_blocks_workspace_size(const harp_plan_t *plan, int64_t n, size_t *bytes) {
  if (!plan || !bytes || n < 0) return HARP_ERR_INVALID_ARG;
  if (plan->col[DIR_FWD].empty()) return HARP_ERR_UNSUPPORTED;
  *bytes = n == 0 ? 0 : grad_workspace_bytes(plan, n);
  return HARP_OK;
}

harp_status_t harp_grad_blocks(const harp_plan_t *plan, const void *X, int64_t ldx, const void *G,
                               int64_t ldg, int64_t n, harp_dtype_t dt, float *const *dK, void *dX,
                               int64_t lddx, void *workspace, size_t workspace_bytes,
                               void *stream) {
  if (!plan || !dK || n < 0) return HARP_ERR_INVALID_ARG;
  if (dt != HARP_F32 && dt != HARP_BF16) return HARP_ERR_INVALID_ARG;
  for (int t = 0; t < plan->m; ++t)
    if (!dK[t]) return HARP_ERR_INVALID_ARG;
  if (n > 0) {
    if (!X || !G || ldx < plan->d || ldg < plan->d) return HARP_ERR_INVALID_ARG;
    if (dX && lddx < plan->d) return HARP_ERR_INVALID_ARG;
  }
  if (plan->col[DIR_FWD].empty()) return HARP_ERR_UNSUPPORTED;
  size_t need = 0;
  harp_status_t st = harp_grad_blocks_workspace_size(plan, n, &need);
  if (st != HARP_OK) return st;
  if (need > 0 && (!workspace || workspace_bytes < need)) return HARP_ERR_INVALID_ARG;
  return launch_grad(plan, X, ldx, G, ldg, n, dt, dK, dX, lddx, workspace, (hipStream_t)stream);
}

// Largest divisor of r in [2, cap], or 0 when r has none there.  Divisors come in pairs
// (q, r / q) with q <= sqrt(r), so one walk over q sees every one of them.
static int64_t largest_divisor_at_most(int64_t r, int64_t cap) {
  if (r < 2) return 0;
  if (r <= cap) return r;
  int64_t best = 0;
  for (int64_t q = 1; q * q <= r; ++q) {
    if (r % q) continue;
    const int64_t p = r / q;
    if (q >= 2 && q <= cap && q > best) best = q;
    if (p >= 2 && p <= cap && p > best) best = p;
  }
  return best;
}

harp_status_t harp_greedy_schedule(int64_t d, int32_t b_base, int32_t b_max, int32_t *out_radices,
                                   int32_t *out_m) {
  if (!out_radices || !out_m) return HARP_ERR_INVALID_ARG;
  if (d < 2 || b_base < 2 || b_max < 2) return HARP_ERR_INVALID_ARG;
  if (d > ((int64_t)1 << 40)) return HARP_ERR_UNSUPPORTED;   // keeps the divisor search short
  // What the appendix's schedule procedure produces, stated as a property: b_base with its
  // full multiplicity in d; then, of what remains, again and again the largest divisor that
  // does not exceed b_max (the sequence is non-increasing because the divisors of a quotient
  // are divisors of the number); a remainder without such a divisor becomes one last stage.
  std::vector<int64_t> sched;
  int64_t r = d;
  while (r % b_base == 0) {
    sched.push_back(b_base);
    r /= b_base;
  }
  for (int64_t f = largest_divisor_at_most(r, b_max); f != 0; f = largest_divisor_at_most(r, b_max)) {
    sched.push_back(f);
    r /= f;
  }
  if (r != 1) sched.push_back(r);
  if (sched.size() > (size_t)HARP_MAX_STAGES) return HARP_ERR_UNSUPPORTED;
  for (int64_t f : sched)
    if (f > INT32_MAX) return HARP_ERR_UNSUPPORTED;
  for (size_t i = 0; i < sched.size(); ++i) out_radices[i] = (int32_t)sched[i];
  *out_m = (int32_t)sched.size();
  return HARP_OK;
}

int64_t harp_plan_dim(const harp_plan_t *plan) { return plan ? plan->d : -1; }
int32_t harp_plan_tied_slices(const harp_plan_t *plan) { return plan ? plan->tied_K : -1; }
int32_t harp_plan_num_stages(const harp_plan_t *plan) { return plan ? plan->m : -1; }
int32_t harp_plan_theta_in_kernel(const harp_plan_t *plan) {
  return plan ? (plan->theta_in_kernel ? 1 : 0) : -1;
}

int64_t harp_plan_param_count(const harp_plan_t *plan) {
  if (!plan) return -1;
  int64_t tot = 0;
  for (int32_t b : plan->radices) tot += (plan->d / b) * ((int64_t)b * (b - 1) / 2);
  return tot;
}

int64_t harp_plan_param_bytes(const harp_plan_t *plan) {
  if (!plan) return -1;
  const HostProgram *hp = select_program(plan, DIR_FWD, (int64_t)1 << 20, nullptr);
  return hp ? hp->param_bytes : -1;
}

harp_status_t harp_plan_set_algo(harp_plan_t *plan, harp_algo_t algo) {
  if (!plan) return HARP_ERR_INVALID_ARG;
  if (algo != HARP_ALGO_AUTO && algo != HARP_ALGO_GENERIC && algo != HARP_ALGO_FUSED &&
      algo != HARP_ALGO_SPLIT)
    return HARP_ERR_INVALID_ARG;
  if (algo != HARP_ALGO_AUTO && !(plan->prog[algo][0].ok && plan->prog[algo][1].ok))
    return HARP_ERR_UNSUPPORTED;
  plan->algo = algo;
  return HARP_OK;
}

harp_status_t harp_plan_set_rows_per_tile(harp_plan_t *plan, int32_t rows) {
  if (!plan || rows < 0) return HARP_ERR_INVALID_ARG;
  plan->rows_override = rows;
  return HARP_OK;
}

const char *harp_plan_kernel_name(const harp_plan_t *plan, int64_t n, harp_dtype_t dt) {
  if (!plan) return "none";
  const char *nm = "none";
  const HostProgram *hp = select_program(plan, DIR_FWD, n, &nm);
  if (hp && hp->n_chunk == hp->prog.npass &&
      dpp_supported(plan, hp->dpp, hp->chunk, nullptr, 8, dt, nullptr, 8, dt))
    return "dpp_radix2";
  if (hp && hp->n_chunk == hp->prog.npass &&
      pipe_supported(plan, hp->prog, 0, hp->prog.npass, hp->chunk, nullptr, 8, nullptr, 8))
    return "pipe_radix2";
  if (hp && hp->n_chunk == hp->prog.npass &&
      wave_supported(plan, hp->prog, 0, hp->prog.npass, hp->chunk, nullptr, 8, nullptr, 8))
    return "wave_radix2";
  if (hp && hp->n_chunk == hp->prog.npass &&
      radix_supported(plan, hp->prog, 0, hp->prog.npass, hp->chunk, nullptr, 8, nullptr, 8))
    return radix_rebuilds_in_kernel(plan, hp->prog, 0, hp->prog.npass, hp->chunk) ? "radix_tile_int8"
                                                                                  : "radix_tile";
  if (hp && hp->n_chunk != hp->prog.npass) {
    const int p0 = hp->chunk_first ? 0 : hp->prog.npass - hp->n_chunk;
    // bf16 callers: the intermediate as block-scaled halves
    if (split_uses_z16(plan, *hp, nullptr, 8, dt, nullptr, 8, dt, n))
      return dpp_supported(plan, hp->dpp, hp->chunk, nullptr, 8, hp->chunk_first ? dt : (harp_dtype_t)kDtZ16,
                           nullptr, 8, hp->chunk_first ? (harp_dtype_t)kDtZ16 : dt)
                 ? "split_dpp_stream_h16"
                 : "split_wave_stream_h16";
    if (pipe_supported(plan, hp->prog, p0, hp->n_chunk, hp->chunk, nullptr, 8, nullptr, 8))
      return "split_pipe_stream";
    if (wave_supported(plan, hp->prog, p0, hp->n_chunk, hp->chunk, nullptr, 8, nullptr, 8))
      return "split_wave_stream";
    if (radix_supported(plan, hp->prog, p0, hp->n_chunk, hp->chunk, nullptr, 8, nullptr, 8))
      return radix_rebuilds_in_kernel(plan, hp->prog, p0, hp->n_chunk, hp->chunk)
                 ? "split_radix_stream_int8"
                 : "split_radix_stream";
  }
  return nm;
}

const char *harp_status_string(harp_status_t status) {
  switch (status) {
    case HARP_OK: return "ok";
    case HARP_ERR_INVALID_ARG: return "invalid argument";
    case HARP_ERR_BAD_SCHEDULE: return "bad schedule (radix < 2, no stages, or product != d)";
    case HARP_ERR_NOT_ORTHOGONAL: return "block is not orthogonal";
    case HARP_ERR_UNSUPPORTED: return "unsupported shape or radix";
    case HARP_ERR_OOM: return "out of memory";
    case HARP_ERR_DEVICE: return "HIP runtime error";
  }
  return "unknown status";
}

const char *harp_version(void) { return "libharp 0.1 (gfx950)"; }

}  // extern "C"
