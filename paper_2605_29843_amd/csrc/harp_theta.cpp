// Parameter front end: block kernels from the rotation parameters Theta (host code, float64).
//
// B_{t,c} = Q(theta_{t,c}) G_{b_t} (block definition of Sec. 3, "Hadamard-preconditioned block
// kernels"): Q is the Givens rotation [[cos, -sin], [sin, cos]] for radix 2 and the Cayley map
// (I + A)^{-1} (I - A) of a skew-symmetric A for larger radices ("Orthogonal parameterization");
// G is the normalised Sylvester Hadamard matrix for power-of-two radices, or a matrix the
// caller supplies.  Theta = 0 gives B = G, i.e. the randomized Hadamard processor for
// power-of-two schedules ("Exact initialization").  The blocks come out in the layout
// harp_plan_create takes.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "harp_internal.h"

namespace {

// normalised Sylvester Hadamard matrix of order b = 2^k: entry (-1)^{popcount(i & j)} / sqrt(b)
void hadamard(int b, std::vector<double> &G) {
  G.assign((size_t)b * b, 0.0);
  const double s = 1.0 / std::sqrt((double)b);
  for (int i = 0; i < b; ++i)
    for (int j = 0; j < b; ++j) G[(size_t)i * b + j] = (__builtin_popcount(i & j) & 1) ? -s : s;
}

// Q = (I + A)^{-1} (I - A) for the skew-symmetric A whose strict upper triangle, row by row,
// is `upper`: Gaussian elimination with partial pivoting on [I + A | I - A].  I + A is always
// invertible (the spectrum of A is imaginary).  Returns false only on a non-finite input.
bool cayley(const float *upper, int b, std::vector<double> &Q, std::vector<double> &work) {
  const int w = 2 * b;
  work.assign((size_t)b * w, 0.0);
  int k = 0;
  for (int i = 0; i < b; ++i) {
    work[(size_t)i * w + i] = 1.0;
    work[(size_t)i * w + b + i] = 1.0;
  }
  for (int i = 0; i < b; ++i)
    for (int j = i + 1; j < b; ++j) {
      const double a = (double)upper[k++];
      if (!std::isfinite(a)) return false;
      work[(size_t)i * w + j] += a;       // I + A
      work[(size_t)j * w + i] -= a;
      work[(size_t)i * w + b + j] -= a;   // I - A
      work[(size_t)j * w + b + i] += a;
    }
  for (int c = 0; c < b; ++c) {
    int piv = c;
    for (int r = c + 1; r < b; ++r)
      if (std::fabs(work[(size_t)r * w + c]) > std::fabs(work[(size_t)piv * w + c])) piv = r;
    if (work[(size_t)piv * w + c] == 0.0) return false;
    if (piv != c)
      for (int j = 0; j < w; ++j) std::swap(work[(size_t)c * w + j], work[(size_t)piv * w + j]);
    const double inv = 1.0 / work[(size_t)c * w + c];
    for (int j = c; j < w; ++j) work[(size_t)c * w + j] *= inv;
    for (int r = 0; r < b; ++r) {
      if (r == c) continue;
      const double f = work[(size_t)r * w + c];
      if (f == 0.0) continue;
      for (int j = c; j < w; ++j) work[(size_t)r * w + j] -= f * work[(size_t)c * w + j];
    }
  }
  Q.resize((size_t)b * b);
  for (int i = 0; i < b; ++i)
    for (int j = 0; j < b; ++j) Q[(size_t)i * b + j] = work[(size_t)i * w + b + j];
  return true;
}

harp_status_t check_schedule(int64_t d, int32_t m, const int32_t *radices) {
  if (!radices) return HARP_ERR_INVALID_ARG;
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
    if (radices[t] > HARP_MAX_RADIX) return HARP_ERR_UNSUPPORTED;
  return HARP_OK;
}

}  // namespace

extern "C" {

harp_status_t harp_blocks_from_theta(int64_t d, int32_t m, const int32_t *radices,
                                     const float *const *theta, const int32_t *mixer_kinds,
                                     const float *const *mixers, float *const *blocks_out) {
  harp_status_t st = check_schedule(d, m, radices);
  if (st != HARP_OK) return st;
  if (!blocks_out) return HARP_ERR_INVALID_ARG;
  for (int t = 0; t < m; ++t) {
    if (!blocks_out[t]) return HARP_ERR_INVALID_ARG;
    const int b = radices[t];
    const int kind = mixer_kinds ? mixer_kinds[t] : HARP_MIXER_HADAMARD;
    if (kind != HARP_MIXER_IDENTITY && kind != HARP_MIXER_HADAMARD && kind != HARP_MIXER_CUSTOM)
      return HARP_ERR_INVALID_ARG;
    if (kind == HARP_MIXER_HADAMARD && (b & (b - 1))) return HARP_ERR_INVALID_ARG;
    if (kind == HARP_MIXER_CUSTOM && (!mixers || !mixers[t])) return HARP_ERR_INVALID_ARG;
  }
  try {
    std::vector<double> G, Q, work;
    for (int t = 0; t < m; ++t) {
      const int b = radices[t];
      const int64_t D = d / b;
      const int npar = b * (b - 1) / 2;
      const int kind = mixer_kinds ? mixer_kinds[t] : HARP_MIXER_HADAMARD;
      if (kind == HARP_MIXER_HADAMARD) {
        hadamard(b, G);
      } else if (kind == HARP_MIXER_IDENTITY) {
        G.assign((size_t)b * b, 0.0);
        for (int i = 0; i < b; ++i) G[(size_t)i * b + i] = 1.0;
      } else {
        G.resize((size_t)b * b);
        for (int i = 0; i < b * b; ++i) G[i] = (double)mixers[t][i];
      }
      const float *th = theta ? theta[t] : nullptr;
      float *out = blocks_out[t];
      for (int64_t c = 0; c < D; ++c) {
        float *K = out + (size_t)c * b * b;
        if (!th) {
          for (int i = 0; i < b * b; ++i) K[i] = (float)G[i];
          continue;
        }
        if (b == 2) {
          const double a = (double)th[c];
          if (!std::isfinite(a)) return HARP_ERR_INVALID_ARG;
          const double cs = std::cos(a), sn = std::sin(a);
          Q.assign({cs, -sn, sn, cs});
        } else if (!cayley(th + (size_t)c * npar, b, Q, work)) {
          return HARP_ERR_INVALID_ARG;
        }
        for (int i = 0; i < b; ++i)
          for (int j = 0; j < b; ++j) {
            double acc = 0.0;
            for (int k = 0; k < b; ++k) acc += Q[(size_t)i * b + k] * G[(size_t)k * b + j];
            K[(size_t)i * b + j] = (float)acc;
          }
      }
    }
  } catch (const std::bad_alloc &) {
    return HARP_ERR_OOM;
  }
  return HARP_OK;
}

harp_status_t harp_plan_create_from_theta(harp_plan_t **out, int64_t d, int32_t m,
                                          const int32_t *radices, const float *const *theta,
                                          const int32_t *mixer_kinds, const float *const *mixers,
                                          const int8_t *signs, uint32_t flags) {
  if (!out) return HARP_ERR_INVALID_ARG;
  if (flags & HARP_BLOCKS_ON_DEVICE) return HARP_ERR_INVALID_ARG;   // Theta is read on the host
  harp_status_t st = check_schedule(d, m, radices);
  if (st != HARP_OK) return st;
  if (d > (int64_t)1 << 24) return HARP_ERR_UNSUPPORTED;
  try {
    std::vector<std::vector<float>> store((size_t)m);
    std::vector<float *> outp((size_t)m);
    std::vector<const float *> inp((size_t)m);
    for (int t = 0; t < m; ++t) {
      store[t].resize((size_t)d * radices[t]);
      outp[t] = store[t].data();
      inp[t] = store[t].data();
    }
    st = harp_blocks_from_theta(d, m, radices, theta, mixer_kinds, mixers, outp.data());
    if (st != HARP_OK) return st;
    return harp_plan_create(out, d, m, radices, inp.data(), signs, flags);
  } catch (const std::bad_alloc &) {
    return HARP_ERR_OOM;
  }
}

// Int8 storage of the stage parameters (appendix "Int8 storage of HARP parameters"): per block
// a scale s = max|a| / 127 over its b(b-1)/2 parameters (the one Givens angle for radix 2) and
// codes q = round(a / s).  The decision is taken in float32 with ties to even; a block whose
// parameters are all zero gets s = 0 and codes 0.
harp_status_t harp_theta_quantize_int8(int64_t d, int32_t m, const int32_t *radices,
                                       const float *const *theta, int8_t *const *codes_out,
                                       float *const *scales_out) {
  harp_status_t st = check_schedule(d, m, radices);
  if (st != HARP_OK) return st;
  if (!theta || !codes_out || !scales_out) return HARP_ERR_INVALID_ARG;
  for (int t = 0; t < m; ++t)
    if (!theta[t] || !codes_out[t] || !scales_out[t]) return HARP_ERR_INVALID_ARG;
  for (int t = 0; t < m; ++t) {
    const int b = radices[t];
    const int64_t D = d / b;
    const int npar = b * (b - 1) / 2;
    for (int64_t c = 0; c < D; ++c) {
      const float *a = theta[t] + (size_t)c * npar;
      float amax = 0.0f;
      for (int i = 0; i < npar; ++i) {
        if (!std::isfinite(a[i])) return HARP_ERR_INVALID_ARG;
        amax = std::max(amax, std::fabs(a[i]));
      }
      const float s = amax / 127.0f;
      scales_out[t][c] = s;
      for (int i = 0; i < npar; ++i) {
        float q = 0.0f;
        if (s > 0.0f) q = std::nearbyintf(a[i] / s);   // default rounding mode: ties to even
        if (!(q >= -127.0f)) q = -127.0f;              // also catches a quotient that overflowed
        if (!(q <= 127.0f)) q = 127.0f;
        codes_out[t][(size_t)c * npar + i] = (int8_t)q;
      }
    }
  }
  return HARP_OK;
}

// a = s * q in float32, the run-time reconstruction of the same appendix.
harp_status_t harp_theta_dequantize_int8(int64_t d, int32_t m, const int32_t *radices,
                                         const int8_t *const *codes, const float *const *scales,
                                         float *const *theta_out) {
  harp_status_t st = check_schedule(d, m, radices);
  if (st != HARP_OK) return st;
  if (!codes || !scales || !theta_out) return HARP_ERR_INVALID_ARG;
  for (int t = 0; t < m; ++t)
    if (!codes[t] || !scales[t] || !theta_out[t]) return HARP_ERR_INVALID_ARG;
  for (int t = 0; t < m; ++t) {
    const int b = radices[t];
    const int64_t D = d / b;
    const int npar = b * (b - 1) / 2;
    for (int64_t c = 0; c < D; ++c) {
      const float s = scales[t][c];
      if (!std::isfinite(s) || s < 0.0f) return HARP_ERR_INVALID_ARG;
      for (int i = 0; i < npar; ++i) {
        const int8_t q = codes[t][(size_t)c * npar + i];
        if (q == -128) return HARP_ERR_INVALID_ARG;   // not a code the quantizer produces
        theta_out[t][(size_t)c * npar + i] = s * (float)q;
      }
    }
  }
  return HARP_OK;
}

harp_status_t harp_plan_create_from_theta_int8(harp_plan_t **out, int64_t d, int32_t m,
                                               const int32_t *radices, const int8_t *const *codes,
                                               const float *const *scales,
                                               const int32_t *mixer_kinds,
                                               const float *const *mixers, const int8_t *signs,
                                               uint32_t flags) {
  if (!out) return HARP_ERR_INVALID_ARG;
  if (flags & HARP_BLOCKS_ON_DEVICE) return HARP_ERR_INVALID_ARG;   // codes are read on the host
  const bool in_kernel = (flags & HARP_THETA_IN_KERNEL) != 0;
  flags &= ~(uint32_t)HARP_THETA_IN_KERNEL;
  harp_status_t st = check_schedule(d, m, radices);
  if (st != HARP_OK) return st;
  if (d > (int64_t)1 << 24) return HARP_ERR_UNSUPPORTED;
  try {
    std::vector<std::vector<float>> store((size_t)m);
    std::vector<float *> outp((size_t)m);
    std::vector<const float *> inp((size_t)m);
    for (int t = 0; t < m; ++t) {
      store[t].resize((size_t)(d / radices[t]) * (radices[t] * (radices[t] - 1) / 2));
      outp[t] = store[t].data();
      inp[t] = store[t].data();
    }
    st = harp_theta_dequantize_int8(d, m, radices, codes, scales, outp.data());
    if (st != HARP_OK) return st;
    st = harp_plan_create_from_theta(out, d, m, radices, inp.data(), mixer_kinds, mixers, signs,
                                     flags);
    if (st != HARP_OK || !in_kernel) return st;
    st = harp::plan_attach_theta_int8(*out, codes, scales, mixer_kinds, signs);
    if (st != HARP_OK) {
      harp_plan_destroy(*out);
      *out = nullptr;
    }
    return st;
  } catch (const std::bad_alloc &) {
    return HARP_ERR_OOM;
  }
}

harp_status_t harp_kronecker_blocks(int32_t K, const float *table, int64_t n2, int32_t m2,
                                    const int32_t *radices2, const float *const *blocks2,
                                    int32_t *radices_out, float *const *blocks_out) {
  if (!table || !blocks2 || !radices_out || !blocks_out) return HARP_ERR_INVALID_ARG;
  if (K < 2) return HARP_ERR_INVALID_ARG;
  harp_status_t st = check_schedule(n2, m2, radices2);
  if (st != HARP_OK) return st;
  if (K > HARP_MAX_RADIX || m2 + 1 > HARP_MAX_STAGES) return HARP_ERR_UNSUPPORTED;
  for (int t = 0; t < m2; ++t)
    if (!blocks2[t] || !blocks_out[t]) return HARP_ERR_INVALID_ARG;
  if (!blocks_out[m2]) return HARP_ERR_INVALID_ARG;
  // the table must be Hadamard-like: entries +-1 and H H^T = K I
  for (int i = 0; i < K * K; ++i)
    if (table[i] != 1.0f && table[i] != -1.0f) return HARP_ERR_INVALID_ARG;
  for (int i = 0; i < K; ++i)
    for (int j = 0; j < K; ++j) {
      int acc = 0;
      for (int k = 0; k < K; ++k) acc += (int)table[i * K + k] * (int)table[j * K + k];
      if (acc != (i == j ? K : 0)) return HARP_ERR_NOT_ORTHOGONAL;
    }
  for (int t = 0; t < m2; ++t) {
    const int b = radices2[t];
    const size_t per = (size_t)(n2 / b) * b * b;   // one copy of the stage's blocks
    radices_out[t] = b;
    for (int k = 0; k < K; ++k)
      for (size_t i = 0; i < per; ++i) blocks_out[t][(size_t)k * per + i] = blocks2[t][i];
  }
  radices_out[m2] = K;
  const double s = 1.0 / std::sqrt((double)K);
  for (int64_t c = 0; c < n2; ++c)
    for (int i = 0; i < K * K; ++i) blocks_out[m2][(size_t)c * K * K + i] = (float)(table[i] * s);
  return HARP_OK;
}

harp_status_t harp_plan_create_kronecker(harp_plan_t **out, int32_t K, const float *table,
                                         int64_t n2, int32_t m2, const int32_t *radices2,
                                         const float *const *blocks2, const int8_t *signs,
                                         uint32_t flags) {
  if (!out || !table || !radices2 || !blocks2) return HARP_ERR_INVALID_ARG;
  if (flags & ~(uint32_t)(HARP_VALIDATE_ORTHO | HARP_F32_INTERMEDIATES)) return HARP_ERR_INVALID_ARG;
  if (K < 2 || n2 < 2 || m2 < 1) return HARP_ERR_INVALID_ARG;
  if (K > HARP_MAX_RADIX || m2 + 1 > HARP_MAX_STAGES) return HARP_ERR_UNSUPPORTED;
  if (n2 > ((int64_t)1 << 24) / K) return HARP_ERR_UNSUPPORTED;
  harp_status_t st = check_schedule(n2, m2, radices2);
  if (st != HARP_OK) return st;
  try {
    // the equivalent Mixed-Radix processor (host copies of every slice's blocks: what the oracle
    // and the untied kernels consume; the tied plan keeps one slice's image on the device)
    std::vector<int32_t> radices(m2 + 1);
    std::vector<std::vector<float>> store(m2 + 1);
    std::vector<float *> outs(m2 + 1);
    for (int t = 0; t < m2; ++t) store[t].resize((size_t)K * n2 * radices2[t]);
    store[m2].resize((size_t)n2 * K * K);
    for (int t = 0; t <= m2; ++t) outs[t] = store[t].data();
    st = harp_kronecker_blocks(K, table, n2, m2, radices2, blocks2, radices.data(), outs.data());
    if (st != HARP_OK) return st;
    std::vector<const float *> blk(outs.begin(), outs.end());
    const int64_t d = (int64_t)K * n2;
    st = harp::plan_create_impl(out, d, m2 + 1, radices.data(), blk.data(), signs, flags, K);
    // no kernel reads a tied image for this shape (slices other than 256 / 512 / 1024 radix-2
    // coordinates, a table below order 9, blocks outside the two-shear form): the expansion
    if (st == HARP_ERR_UNSUPPORTED)
      st = harp::plan_create_impl(out, d, m2 + 1, radices.data(), blk.data(), signs, flags, 0);
    return st;
  } catch (const std::bad_alloc &) {
    return HARP_ERR_OOM;
  }
}

}  // extern "C"
