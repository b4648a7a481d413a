// Internal descriptors shared between the host planner and the HIP kernels of libmona.
// Nothing here is part of the public ABI (see include/mona.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>

namespace mona {

typedef __bf16 bf16_t;

// Static per-matrix description, uploaded once when the state is built.
struct MatStatic {
  void* g_prev;        // G_{k-1}, state dtype (NULL in the one-buffer form and when the caller keeps it)
  void* acc;           // A_k (or, in the one-buffer form, C_{k+1}), state dtype
  float* mom;          // M_k, fp32
  void* x;             // where the Newton-Schulz input (M_k, unscaled) is written: bf16 or fp32
  int32_t m, n;        // shape
  int32_t ldx;         // leading dimension of x (>= n)
  int32_t w_dtype, g_dtype;
  int32_t first_block; // first block of the elementwise grid that belongs to this matrix
  int32_t num_blocks;  // number of such blocks
  int32_t x_f32;       // 1: x (and the whole Newton-Schulz workspace of this matrix) is fp32, else bf16
};

// Per-step pointers (the caller may pass fresh buffers every step).
struct MatDynamic {
  void* w;
  const void* g;
  void* slot;          // caller-kept G_{k-1} (streaming variant), else NULL
};

// Result of the per-matrix Frobenius norm (Sec. 3.2, X_0 = M / ||M||_F).
struct MatScale {
  float inv;        // 1 / (||M||_F + eps) for the working copy as it stands (see xexp), 0 when the
                    // denominator is 0 or not finite
  float inv2;       // inv * inv
  float norm;       // ||M||_F
  uint32_t status;  // MONA_STATUS_* bits
  int32_t xexp;     // the working copy holds M 2^xexp (0 unless the norm left the safe window)
};

// One entry per block of the elementwise grid.
struct BlockWork {
  int32_t mat;    // matrix index
  int32_t chunk;  // chunk index inside that matrix
};

constexpr int kEwThreads = 256;
constexpr int kEwChunk = 4096;  // elements per block of the elementwise kernel

// ---- Newton-Schulz product kernels -------------------------------------------------
// out = post * (beta * E + alpha * (P Q^T)) + diag * I,   P: M x K,  Q: N x K  (logical shapes)
// An operand flagged "transposed" is stored K-major (K x M or K x N, rows of length ld).
enum GemmEpilogue : int32_t {
  EPI_STORE = 0,   // store `out`
  EPI_UPDATE = 1,  // `out` is O_k: apply W <- (1 - eta lambda) W - eta gamma O, optionally store O
};

enum PostScale : int32_t { POST_NONE = 0, POST_INV = 1, POST_INV2 = 2 };

struct GemmArgs {
  const void* P; const void* Q; const void* E; void* C;
  int64_t strideP, strideQ, strideE, strideC;  // elements between consecutive matrices of the group
  int32_t ldp, ldq, lde, ldc;
  int32_t M, N, K;          // padded problem size, multiples of the tile
  int32_t tile_m, tile_n;   // BM, BN of the kernel that will run
  int32_t sym_ratio;        // BM / BN (symmetric products walk the block triangle with it)
  int32_t tiles_m, tiles_n; // M / BM, N / BN
  int32_t tiles_per_mat;    // tiles_m * tiles_n, or the triangle count when symmetric
  int32_t count;            // matrices in the group
  int32_t symmetric;        // 1: only tiles with tj >= ti are computed, the result is mirrored
  float alpha, beta;
  float diag;               // added to the main diagonal of the result (symmetric products only)
  int32_t post;             // PostScale, indexed through `members`
  int32_t epilogue;         // GemmEpilogue
  int32_t store_out;        // EPI_UPDATE: also store O
  const int32_t* members;   // group member -> matrix index
  const MatScale* scales;   // per matrix
  const MatStatic* stat;    // per matrix (EPI_UPDATE: real m, n, w dtype)
  const MatDynamic* dyn;    // per matrix (EPI_UPDATE: w pointer)
  float w_keep;             // 1 - eta * lambda
  float o_scale;            // eta * gamma
};

// records the text mona_last_error() returns (thread-local) and hands `code` back
int api_fail(int code, const char* fmt, va_list ap);

// kernels (defined in the .hip files)
hipError_t launch_state_update(const MatStatic* stat, const MatDynamic* dyn, const BlockWork* work,
                               double* partials, int num_blocks, int g_bf16, int state_bf16, int one_buffer,
                               float mu, float beta_a, float alpha, int use_prev, hipStream_t s);
// norm_finalize_kernel, then rescue_kernel (repairs the working copies of flagged matrices)
// `list` (DEVICE, may be NULL = matrices 0 .. count - 1): the matrix indices to finalise
hipError_t launch_norm_finalize(const MatStatic* stat, const double* partials, MatScale* scales,
                                const int32_t* list, int count, float eps, hipStream_t s);
// tables of a one-matrix state written by a kernel from its arguments (no host copy)
hipError_t launch_single_tables(const MatStatic& ms, const MatDynamic& md, void* o_ptr, MatStatic* stat,
                                MatDynamic* dyn, void** o_ptrs, BlockWork* work, int num_blocks, int32_t* members,
                                int32_t* order, hipStream_t s);
hipError_t launch_plain_update(const MatStatic* stat, const MatDynamic* dyn, const MatScale* scales,
                               const BlockWork* work, int num_blocks, void* const* o_ptrs, float lr, float wd,
                               float gamma_coeff, int store_o, hipStream_t s);
// cu_cap > 0: the persistent large-tile kernel uses at most that many CUs (the rest are busy elsewhere)
hipError_t launch_ns_gemm(const GemmArgs& a, int tile, bool transP, bool transQ, bool f32, int cu_cap,
                          hipStream_t s);
int device_cu_count();
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);

}  // namespace mona
