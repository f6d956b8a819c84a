// Internal structures shared by the host-side plan builder and the HIP launchers.
// Not part of the public interface.
#ifndef HARP_INTERNAL_H_
#define HARP_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <vector>

#include "harp.h"

namespace harp {

// A *pass* is a run of consecutive stages that one thread executes on a register-resident
// sub-tensor of the row: the P = prod(radices of the run) coordinates
//     base + j * S,  j = 0..P-1,   base = hi * P * S + lo,   q = hi * S + lo  (q < d / P)
// where S is the stride of the run's lowest digit.  Between passes the row tile lives in LDS.
enum PassKind : int32_t {
  PASS_POW2_DENSE = 0,    // k radix-2 stages, 4 values per 2x2 block
  PASS_POW2_LIFT = 1,     // k radix-2 stages, orthogonal blocks as 3 lifting steps: 2 values
  PASS_SMALL = 2,         // one stage of radix 3..8, compile-time radix, block in registers
  PASS_GENERIC = 3,       // one stage of any radix <= HARP_MAX_RADIX, run-time radix
  PASS_POW2_LIFT_LD = 4,  // as LIFT, but the k-th stage (the program's last) is a dense 2x2
  // k radix-2 stages as two shears with deferred output scales, 2 values (f0, f1) per pair:
  // (x0, x1) <- (x0 + f0 x1, x1 + f1 x0); _LD: the k-th stage is the program's dense last one
  PASS_POW2_SCALED = 5,
  PASS_POW2_SCALED_LD = 6,
  // k = 2 consecutive radix-3 stages (adjacent digits) of a split program's streamed part
  // in one trip: P = 3^k coordinates per sub-tensor, value ((e * 3^(k-1) + o) * 9 + r * 3 + r2)
  // = entry [r][r2] of the block that the e-th stage in execution order uses for the
  // combination o of the other digits (ascending); desc = 1: the stages run from the highest
  // digit down
  PASS_SMALL_CHAIN = 7
};

struct PassDesc {
  int32_t kind;
  int32_t b;     // radix of the stage (SMALL / GENERIC); 2 for POW2
  int32_t k;     // number of stages in the pass (POW2), else 1
  int32_t desc;  // POW2: 1 = digits executed from the highest to the lowest (transpose program)
  int32_t P;     // coordinates per sub-tensor
  int32_t S;     // stride of the lowest digit of the pass
  int32_t nq;    // d / P sub-tensors per row
  int32_t V;     // parameter values per sub-tensor
  // Sub-tensors in the parameter image: nq, or -- in a plan with tied parameters (the Kronecker
  // fallback, Eq. (12): every slice of n2 coordinates shares one T_{n2}, and all blocks of the
  // last stage are one table) -- the n2 / P sub-tensors of one slice (a power of two; sub-tensor
  // q reads entry q mod nqp), or 1 for the shared table.
  int32_t nqp;
  int32_t tied;  // 1: parameters indexed modulo nqp
  const float *params;  // device, [V][nqp]: value v of sub-tensor q at params[v * nqp + q mod nqp]
  // GENERIC, radix >= 9: the blocks as bf16 hi/lo MFMA operand tiles of all sub-tensors,
  // followed by the same tiles in float32; SMALL, radix 4 / 8: a
  // second copy of params, four values per 16-byte load ([V/4][nq][4] floats); else null
  const void *aux;
  // SMALL, radix 4 / 8, plans created with HARP_THETA_IN_KERNEL: the stage's int8 image (device)
  // or null.  Radix 8: 16-byte piece k < 2 of block c at ((k * nq) + c) * 16 bytes -- the 28 codes
  // of the strict upper triangle row by row, then one byte of sign bits (bit r set: coordinate r
  // of the block carries a -1 sign; stage 0 only), three bytes of padding -- followed by nq
  // float32 scales.  Radix 4: one 8-byte piece per block (6 codes, sign bits, padding), then the
  // scales.  q8_flags bit 0: Hadamard mixer (else identity), bit 1: apply the sign bits.
  const void *q8;
  int32_t q8_flags;
  int32_t q8_pad;
};

constexpr int kMaxPasses = HARP_MAX_STAGES;

struct Program {
  int32_t npass;
  int32_t reserved;
  PassDesc pass[kMaxPasses];
};

// Execution plan of a program.  Unsplit: every pass runs on the on-chip row tile (chunk == d).
// Split ("four-step"): the passes on the low digits (product `chunk` <= 4096) run fused on chip
// on contiguous chunks of every row; each pass on the digits above is streamed through device
// memory with a float32 intermediate.  In the forward program the chunk passes come first
// ([0, n_chunk)), in the transposed program last ([npass - n_chunk, npass)).
// Parameter image of the two-group DPP kernel (harp_dpp.hip) for the chunk-local radix-2 stages
// of a program, all in the two-shear form (the program's last stage, if among them, dense).
// Per chunk and group: stage e (execution order), 16-byte piece k, thread t, value q at
// ((e * 4 + k) * 256 + t) * 4 + q = the factor of coordinate 16 * segment(t) + 4 k + q; the dense
// stage takes two such slots (own-coordinate factors, then partner factors).
struct DppImage {
  const float *img = nullptr;   // device; null: the program has no such image
  int64_t host_off = -1;        // offset (floats) inside the program's host image, -1: none
  int64_t offB = 0;             // group B's part starts here (floats)
  int64_t strideA = 0, strideB = 0;   // floats per chunk
  bool trn = false, ld = false;
  int32_t logd = 12;            // log2 of the chunk: 12, or 11 (eleven stages, 128 threads per group)
  // transposed split program whose streamed stage (dense, radix topB = 3 or 5, on the digit
  // above the chunk) is executed on the way in (harp_dpp_top_kernel): its factors per output
  // chunk kch, input chunk j, piece k, thread t at offT + (((kch * topB + j) * 4 + k) * 256 + t) * 4
  int32_t topB = 0;
  int64_t offT = 0;
};

struct HostProgram {
  DppImage dpp;
  Program prog{};
  const Program *dev = nullptr;  // device copy of prog (what the kernels read)
  int64_t param_bytes = 0;
  bool ok = false;  // false: some stage has no code path in this family
  int32_t chunk = 0;      // coordinates per on-chip chunk (== d when unsplit)
  int32_t n_chunk = 0;    // number of chunk-local passes
  bool chunk_first = true;
  // split program of a row that also fits one chunk (radix-2 stages + one radix-3 stage): it
  // only pays for large forward batches, see select_program
  bool optional = false;
  // the float32 intermediate may be replaced by block-scaled halves for bf16 callers (set by the
  // plan builder: orthogonal blocks, no scale pending where the intermediate is written)
  bool z16 = false;
};

enum Direction { DIR_FWD = 0, DIR_TRN = 1 };

// ---- column-mode passes (rotate_weight's plan_U side, harp_col.hip) ----
constexpr int kColMaxOps = 8;
// One step of a pass: a single stage of radix b (k == 1), or k <= 3 consecutive radix-2 stages
// executed on 2^k rows in registers.  sp = in-tile stride (in tile rows) of the step's lowest
// digit; sub-stage e (execution order) acts on digit dp[e] of the 2^k rows; poff[e] = where its
// block values start in the tile's value list (floats).
struct ColOp {
  int32_t b, k, sp, pad;
  int32_t dp[3];
  int32_t poff[3];
};

struct ColPass {
  int32_t nops;
  int32_t P;      // rows per tile
  int32_t S;      // row stride between consecutive tile rows
  int32_t npar;   // block values per tile (padded blocks)
  const float *image;     // device: every stage's dense blocks
  // device, [3][npar]: value e of tile (hi, lo) is image[fix[e] + hi * fa[e] + lo * fb[e]];
  // fa[e] == 0xffffffff marks padding
  const uint32_t *ptab;
  ColOp op[kColMaxOps];
};
struct ColPassHost {
  ColPass pass;
  const ColPass *dev;   // device copy
  std::vector<uint32_t> ptab;
};
// stage of the column-mode image, execution order: dense blocks [d / b][b][b] with the signs
// folded in (device memory)
struct ColStage {
  int32_t b;
  int32_t s;
  const float *blocks;
};



// ---- block-scaled half-precision intermediate of split programs ("Z16") --------------------
// Between the chunk kernel and the one streamed stage of a split program a bf16 caller's rows
// may travel as IEEE half-precision values with one shared power-of-two scale per aligned
// segment of 16 coordinates instead of float32: a row of the buffer is d halves followed by
// d / 16 exponent bytes (row pitch z16_ld(d) halves).  Byte e of a segment is the biased
// float32 exponent of its largest magnitude (at most 253); a stored half h stands for
// h * 2^(e - 127), so the largest element of a segment is stored in [1, 2) and every element
// with a relative error of at most 2^-12 of itself or 2^-25 of that largest element.
struct zh16 {
  uint16_t v;
};
constexpr int kDtZ16 = 2;   // internal element-type tag next to HARP_F32 / HARP_BF16
inline int64_t z16_ld(int64_t d) { return (d + d / 32 + 7) / 8 * 8; }

#if defined(__HIPCC__)
__device__ __forceinline__ uint32_t z16_exponent(float largest_magnitude) {
  const uint32_t e = (__float_as_uint(largest_magnitude) >> 23) & 0xffu;
  return e > 253u ? 253u : e;
}
__device__ __forceinline__ float z16_down(uint32_t e) { return __uint_as_float((254u - e) << 23); }
__device__ __forceinline__ float z16_up(uint32_t e) { return __uint_as_float(e << 23); }
__device__ __forceinline__ uint32_t z16_pack(float a, float b) {
  typedef float f2v __attribute__((ext_vector_type(2)));
  typedef _Float16 h2v __attribute__((ext_vector_type(2)));
  const f2v v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, h2v));
}
__device__ __forceinline__ void z16_unpack(uint32_t w, float scale, float &a, float &b) {
  typedef float f2v __attribute__((ext_vector_type(2)));
  typedef _Float16 h2v __attribute__((ext_vector_type(2)));
  const f2v v = __builtin_convertvector(__builtin_bit_cast(h2v, w), f2v);
  a = v.x * scale;
  b = v.y * scale;
}
#endif

struct LaunchCfg {
  int rows_per_tile;
  int threads;
};

}  // namespace harp

struct harp_plan {
  int64_t d = 0;
  int32_t m = 0;
  std::vector<int32_t> radices;
  std::vector<int64_t> strides;
  harp::HostProgram prog[4][2];   // [algo (1 = generic, 2 = fused, 3 = split)][direction]
  std::vector<void *> dev_allocs;
  int algo = HARP_ALGO_AUTO;
  int rows_override = 0;
  int device = 0;
  int lds_bytes = 0;   // usable LDS per workgroup
  int num_cu = 0;
  // float32 intermediates of split programs, one per stream the plan has been used on (work
  // on one stream is ordered, so consecutive calls can share the buffer).  Nothing is freed
  // before the plan is destroyed: a buffer that a later, larger call outgrows moves to
  // `retired`, because launches already queued and HIP graphs captured earlier still hold
  // its address.
  struct Scratch {
    hipStream_t stream;
    float *ptr;
    size_t bytes;
  };
  mutable std::mutex scratch_mu;
  mutable std::vector<Scratch> scratch;
  mutable std::vector<void *> retired;
  bool no_mfma = false;   // HARP_NO_MFMA was set when the plan was created
  // Kronecker plan with tied parameters (harp_plan_create_kronecker): K slices of n2 coordinates;
  // 0: an ordinary plan.  Such a plan has the split program only (wave kernel on the slices +
  // matrix-core stage for the table); the signs are applied inside the wave kernel.
  int32_t tied_K = 0;
  int64_t tied_n2 = 0;
  // column-mode image (every plan) and passes (empty when some radix exceeds 8) per direction
  std::vector<harp::ColStage> col[2];
  // gradient path, stages of radix 9..64 whose stride is a multiple of 16: the blocks of
  // col[DIR_FWD][t] ([0][t]) and their transposes ([1][t]) as matrix-core operand tiles
  // (aux == nullptr: none)
  std::vector<harp::PassDesc> grad_mfma[2];
  std::vector<harp::ColPassHost> colpass[2];
  const int8_t *dev_signs = nullptr;   // device copy of the signs (null: all +1)
  bool orthogonal = true;              // every block satisfies |K^T K - I| <= 1e-5
  bool f32_only = false;               // HARP_F32_INTERMEDIATES: no block-scaled half intermediates
  bool theta_in_kernel = false;        // some pass carries an int8 image (HARP_THETA_IN_KERNEL)
};

namespace harp {

// launchers (harp_kernels.hip)
// passes [p0, p1) of the program on row chunks of `chunk` coordinates (chunk == d: whole rows)
harp_status_t launch_tile_kernel(const harp_plan *plan, const Program *dev_prog, int p0, int p1,
                                 int chunk, const void *X, int64_t ldx, harp_dtype_t dt_in,
                                 void *Y, int64_t ldy, harp_dtype_t dt_out, int64_t n,
                                 hipStream_t stream);
// one pass streamed through device memory (sub-tensor per thread, parameters in registers)
// allow_narrow: the caller's element type is bf16, so large-radix passes may use the MFMA
// kernel with bf16-split operands
harp_status_t launch_stream_pass(const harp_plan *plan, const HostProgram &hp, int p,
                                 const void *X, int64_t ldx, harp_dtype_t dt_in, void *Y,
                                 int64_t ldy, harp_dtype_t dt_out, int64_t n, bool allow_narrow,
                                 hipStream_t stream);
bool stream_z16_supported(const PassDesc &pd, const void *X, int64_t ldx, const void *Y,
                          int64_t ldy);
// large-radix stage on the matrix cores (harp_mfma.hip)
bool mfma_pass_supported(const PassDesc &pd, const void *X, int64_t ldx, const void *Y,
                         int64_t ldy);
harp_status_t launch_mfma_pass(const harp_plan *plan, const PassDesc &pd, const void *X,
                               int64_t ldx, harp_dtype_t dt_in, void *Y, int64_t ldy,
                               harp_dtype_t dt_out, int64_t n, bool narrow, hipStream_t stream);
harp_status_t launch_transpose(const void *src, int64_t lds_, harp_dtype_t dt_src, void *dst,
                               int64_t ldd, harp_dtype_t dt_dst, int64_t rows, int64_t cols,
                               hipStream_t stream);
harp_status_t launch_copy2d(const void *src, int64_t lds_, void *dst, int64_t ldd, int64_t rows,
                            int64_t cols, harp_dtype_t dt, hipStream_t stream);
LaunchCfg choose_launch(const harp_plan *plan, int64_t chunk, int64_t nrows);
// row-pipelined radix-2 kernel (harp_pipe.hip): passes [p0, p0+np) on chunks of `chunk`
bool pipe_supported(const harp_plan *plan, const Program &prog, int p0, int np, int chunk,
                    const void *X, int64_t ldx, const void *Y, int64_t ldy);
harp_status_t launch_pipe_kernel(const harp_plan *plan, const HostProgram &hp, int p0, int chunk,
                                 const void *X, int64_t ldx, harp_dtype_t dt_in, void *Y,
                                 int64_t ldy, harp_dtype_t dt_out, int64_t n, int rows_per_tile,
                                 hipStream_t stream);
// two-group DPP kernel for radix-2 chains in the two-shear form on chunks of 4096 (harp_dpp.hip)
unsigned dpp_segment_of(bool high_layout, unsigned t, int logd = 12);
bool dpp_supported(const harp_plan *plan, const DppImage &di, int chunk, const void *X, int64_t ldx,
                   harp_dtype_t dt_in, const void *Y, int64_t ldy, harp_dtype_t dt_out);
harp_status_t launch_dpp_kernel(const harp_plan *plan, const DppImage &di, const void *X,
                                int64_t ldx, harp_dtype_t dt_in, void *Y, int64_t ldy,
                                harp_dtype_t dt_out, int64_t n, int rows_per_tile,
                                hipStream_t stream);
bool dpp_top_supported(const harp_plan *plan, const DppImage &di, const void *X, int64_t ldx,
                       harp_dtype_t dt_in, const void *Y, int64_t ldy, harp_dtype_t dt_out);
harp_status_t launch_dpp_top_kernel(const harp_plan *plan, const DppImage &di, const void *X,
                                    int64_t ldx, void *Y, int64_t ldy, int64_t n, int rows_per_tile,
                                    hipStream_t stream);
// wave-local radix-2 kernel for chunks of 256 / 512 / 1024 coordinates (harp_pipe.hip)
bool wave_supported(const harp_plan *plan, const Program &prog, int p0, int np, int chunk,
                    const void *X, int64_t ldx, const void *Y, int64_t ldy);
harp_status_t launch_wave_kernel(const harp_plan *plan, const HostProgram &hp, int p0, int np,
                                 int chunk, const void *X, int64_t ldx, harp_dtype_t dt_in,
                                 void *Y, int64_t ldy, harp_dtype_t dt_out, int64_t n,
                                 hipStream_t stream);
// extern "C" body of harp_plan_create with the Kronecker tying as an extra argument (harp_api.cpp)
harp_status_t plan_create_impl(harp_plan **out, int64_t d, int32_t m, const int32_t *radices,
                               const float *const *blocks, const int8_t *signs, uint32_t flags,
                               int32_t tied_K);
// Attach the int8 images of the stages that have a run-time reconstruction kernel (equal-radix
// chains of radix 4 / 8, Hadamard or identity mixer) to a plan built from the same codes
// (harp_api.cpp); returns HARP_OK also when no stage qualifies.
harp_status_t plan_attach_theta_int8(harp_plan *plan, const int8_t *const *codes,
                                     const float *const *scales, const int32_t *mixer_kinds,
                                     const int8_t *signs);
// tile kernel for chains of equal radix 4 or 8 on chunks of 4^m / 8^m coordinates (harp_radix.hip)
bool radix_supported(const harp_plan *plan, const Program &prog, int p0, int np, int chunk,
                     const void *X, int64_t ldx, const void *Y, int64_t ldy);
bool radix_rebuilds_in_kernel(const harp_plan *plan, const Program &prog, int p0, int np, int chunk);
harp_status_t launch_radix_kernel(const harp_plan *plan, const HostProgram &hp, int p0, int np,
                                  int chunk, const void *X, int64_t ldx, harp_dtype_t dt_in,
                                  void *Y, int64_t ldy, harp_dtype_t dt_out, int64_t n,
                                  hipStream_t stream);
// column-mode passes (harp_col.hip): group plan->col[dir] into passes; launch one pass on a
// row-major [nrows, ncols] matrix (nrows == plan->d; may run in place)
bool build_col_passes(const harp_plan *plan, Direction dir, std::vector<ColPassHost> &out);
harp_status_t launch_col_pass(const harp_plan *plan, const ColPass *dpass, const ColPass &hp,
                              const void *src,
                              int64_t lds_, harp_dtype_t dt_src, void *dst, int64_t ldd,
                              harp_dtype_t dt_dst, int64_t nrows, int64_t ncols,
                              hipStream_t stream);
// block-scaled halves (kDtZ16) on either side of a column pass: unguarded tiles only
bool col_z16_supported(const ColPass &hp, const void *src, int64_t lds_, const void *dst,
                       int64_t ldd, int64_t nrows, int64_t ncols);
// a pass of radix-2 stages on 32 / 64 / 128-row tiles that runs with the tile in registers
bool col_pass_in_registers(const ColPass &hp, int64_t ncols);
// column pass fused with the row-side processor's streamed small-radix stage (harp_col.hip)
bool colrow_supported(const harp_plan *plan, const ColPass &hp, const PassDesc &vp, const void *src,
                      int64_t lds_, harp_dtype_t dt_src, const void *dst, int64_t ldd,
                      harp_dtype_t dt_dst, int64_t nrows, int64_t ncols);
harp_status_t launch_colrow_pass(const harp_plan *plan, const ColPass *dpass, const ColPass &hp,
                                 const PassDesc &vp, const void *src, int64_t lds_,
                                 harp_dtype_t dt_src, void *dst, int64_t ldd, harp_dtype_t dt_dst,
                                 int64_t nrows, int64_t ncols, hipStream_t stream);
// gradient with respect to the blocks (harp_grad.hip); needs plan->col[DIR_FWD]
size_t grad_workspace_bytes(const harp_plan *plan, int64_t n);
harp_status_t launch_grad(const harp_plan *plan, const void *X, int64_t ldx, const void *G,
                          int64_t ldg, int64_t n, harp_dtype_t dt, float *const *dK, void *dX,
                          int64_t lddx, void *ws, hipStream_t st);
int choose_pipe_rows(const harp_plan *plan, int64_t n, int64_t nchunk, int chunk);
const HostProgram *select_program(const harp_plan *plan, Direction dir, int64_t n,
                                  const char **name);

}  // namespace harp
#endif
