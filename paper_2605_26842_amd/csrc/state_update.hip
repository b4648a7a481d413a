// Elementwise part of the MONA step (Alg. 1: difference, acceleration EMA, accelerated
// gradient, momentum, state roll) fused with the sum of squares that the Newton-Schulz
// prescale X_0 = M / ||M||_F needs (Sec. 3.2).  One pass over the state: every array is
// read once and written once, 16 bytes per lane, so the kernel runs at HBM speed.
//
// Per element, with fp32 G and fp32 state: reads G, G_{k-1}, A, M (16 B), writes G_{k-1}, A, M
// (12 B) and the bf16 copy of M that the matrix products read (2 B): 30 B.  In the one-buffer form
// (no stored G_{k-1}: the bracket C_k = beta_a A_{k-1} - (1 - beta_a) G_{k-1} is carried instead of
// A and G_{k-1}, and A_k = C_k + (1 - beta_a) G_k) it reads G, C, M and writes C, M and the copy: 22 B.
#include "mona_internal.h"

namespace mona {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));

// The state is streamed: every array is read once and written once per step and is not touched
// again before the next step, so the accesses are marked non-temporal.
template <typename V> __device__ __forceinline__ V stream_load(const V* p) { return __builtin_nontemporal_load(p); }
template <typename V> __device__ __forceinline__ void stream_store(V* p, V v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ f32x4 load4(const float* p) { return stream_load(reinterpret_cast<const f32x4*>(p)); }
__device__ __forceinline__ f32x4 load4(const bf16_t* p) {
  bf16x4 v = stream_load(reinterpret_cast<const bf16x4*>(p));
  f32x4 r = {(float)v.x, (float)v.y, (float)v.z, (float)v.w};
  return r;
}
__device__ __forceinline__ void store4(float* p, f32x4 v) { stream_store(reinterpret_cast<f32x4*>(p), v); }
__device__ __forceinline__ void store4(bf16_t* p, f32x4 v) {
  bf16x4 r = {(bf16_t)v.x, (bf16_t)v.y, (bf16_t)v.z, (bf16_t)v.w};  // round to nearest even
  stream_store(reinterpret_cast<bf16x4*>(p), r);
}
__device__ __forceinline__ float load1(const float* p) { return *p; }
__device__ __forceinline__ float load1(const bf16_t* p) { return (float)*p; }
__device__ __forceinline__ void store1(float* p, float v) { *p = v; }
__device__ __forceinline__ void store1(bf16_t* p, float v) { *p = (bf16_t)v; }

// value the stored state holds after rounding to its dtype (identity for fp32)
template <typename ST> __device__ __forceinline__ float stored(float v) { return v; }
template <> __device__ __forceinline__ float stored<bf16_t>(float v) { return (float)(bf16_t)v; }

struct Coef {
  float mu, beta, one_minus_beta, alpha;
  int use_prev;
};

// One element of Alg. 1's elementwise lines.  Returns M_k; updates a (A_k) in place.
__device__ __forceinline__ float mona_element(float g, float gp, float& a, float m, const Coef& c) {
  float d = c.use_prev ? (g - gp) : 0.0f;            // D_k = G_k - G_{k-1}
  a = c.beta * a + c.one_minus_beta * d;             // A_k = beta_a A_{k-1} + (1 - beta_a) D_k
  float gt = g + c.alpha * a;                        // Gt_k = G_k + alpha A_k
  return c.mu * m + gt;                              // M_k = mu M_{k-1} + Gt_k
}

// The squares are summed in double: M_ij^2 leaves the fp32 range once |M_ij| is below about 1e-19 or above
// 1e19 (a matrix that has received no gradient for a few hundred steps decays to such values), and the
// norm must still come out right there.  The kernel is bound by HBM; the fp64 operations are free.
__device__ __forceinline__ double block_sum(double v, double* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);   // within the wavefront
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[wave] = v;                            // then across wavefronts in LDS
  __syncthreads();
  double t = 0.0;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 0; w < kEwThreads / 64; ++w) t += red[w];
  }
  return t;
}

// One element in the one-buffer form.  c holds C_k on entry and C_{k+1} on return; returns M_k.
// With use_prev == 0 (first step, "G_0 := G_1") A_1 = 0, i.e. C_1 = -(1 - beta_a) G_1.
__device__ __forceinline__ float mona_element_one_buffer(float g, float& cbuf, float m, const Coef& c) {
  const float a = c.use_prev ? (cbuf + c.one_minus_beta * g) : 0.0f;   // A_k
  const float gt = g + c.alpha * a;
  cbuf = c.beta * a - c.one_minus_beta * g;
  return c.mu * m + gt;
}

enum StateMode : int { MODE_MUON = 0, MODE_TWO_BUFFER = 1, MODE_ONE_BUFFER = 2 };

// MODE_MUON is plain Muon (Eq. muon_momentum fed with G_k itself): the acceleration buffers
// are neither read nor written.
template <typename GT, typename ST, int MODE>
__global__ __launch_bounds__(kEwThreads) void state_update_kernel(
    const MatStatic* __restrict__ stat, const MatDynamic* __restrict__ dyn,
    const BlockWork* __restrict__ work, double* __restrict__ partials, Coef c) {
  __shared__ double red[kEwThreads / 64];
  const BlockWork bw = work[blockIdx.x];
  const MatStatic ms = stat[bw.mat];
  const GT* __restrict__ g = static_cast<const GT*>(dyn[bw.mat].g);
  // G_{k-1} lives in the arena, or (streaming variant) in the slot the caller keeps
  ST* __restrict__ gp = static_cast<ST*>(ms.g_prev ? ms.g_prev : dyn[bw.mat].slot);
  ST* __restrict__ ac = static_cast<ST*>(ms.acc);
  float* __restrict__ mo = ms.mom;
  // working copy of M_k for the matrix products: bf16, or fp32 for matrices orthogonalised in fp32
  bf16_t* __restrict__ xh = static_cast<bf16_t*>(ms.x);
  float* __restrict__ xf = static_cast<float*>(ms.x);
  const bool xf32 = ms.x_f32 != 0;

  const int total = ms.m * ms.n;
  const int base = bw.chunk * kEwChunk;
  const int count = min(kEwChunk, total - base);
  const int n = ms.n, ldx = ms.ldx;
  double ss = 0.0;

  if ((n & 3) == 0) {
    // rows are a multiple of 4 elements: 4-element groups never straddle a row
    constexpr int kIter = kEwChunk / (kEwThreads * 4);
    constexpr int kBatch = 4;
    static_assert(kIter % kBatch == 0, "chunk must be a multiple of the batch");
    for (int it0 = 0; it0 < kIter; it0 += kBatch) {
      f32x4 vg[kBatch], vp[kBatch], va[kBatch], vm[kBatch];
      int idx[kBatch];
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        const int i = ((it0 + b) * kEwThreads + threadIdx.x) * 4;
        idx[b] = (i < count) ? base + i : -1;
        if (idx[b] >= 0) {
          vg[b] = load4(g + idx[b]);
          if constexpr (MODE == MODE_TWO_BUFFER) vp[b] = load4(gp + idx[b]);
          if constexpr (MODE != MODE_MUON) va[b] = load4(ac + idx[b]);
          vm[b] = load4(mo + idx[b]);
        }
      }
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        if (idx[b] >= 0) {
          float a4[4] = {0.0f, 0.0f, 0.0f, 0.0f}, p4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
          if constexpr (MODE != MODE_MUON) { a4[0] = va[b].x; a4[1] = va[b].y; a4[2] = va[b].z; a4[3] = va[b].w; }
          if constexpr (MODE == MODE_TWO_BUFFER) { p4[0] = vp[b].x; p4[1] = vp[b].y; p4[2] = vp[b].z; p4[3] = vp[b].w; }
          const float g4[4] = {vg[b].x, vg[b].y, vg[b].z, vg[b].w};
          const float m4[4] = {vm[b].x, vm[b].y, vm[b].z, vm[b].w};
          float n4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if constexpr (MODE == MODE_TWO_BUFFER) n4[e] = mona_element(g4[e], p4[e], a4[e], m4[e], c);
            else if constexpr (MODE == MODE_ONE_BUFFER) n4[e] = mona_element_one_buffer(g4[e], a4[e], m4[e], c);
            else n4[e] = c.mu * m4[e] + g4[e];
          }
          const f32x4 a = {a4[0], a4[1], a4[2], a4[3]};
          const f32x4 mnew = {n4[0], n4[1], n4[2], n4[3]};
          ss += (double)mnew.x * mnew.x + (double)mnew.y * mnew.y + (double)mnew.z * mnew.z + (double)mnew.w * mnew.w;
          if constexpr (MODE == MODE_TWO_BUFFER) store4(gp + idx[b], vg[b]);   // G_{k-1} <- G_k
          if constexpr (MODE != MODE_MUON) store4(ac + idx[b], a);              // A_k, or C_{k+1}
          store4(mo + idx[b], mnew);
          // the padded copy can exceed 2^31 elements although m * n does not: 64-bit offset
          const int64_t xo = (ldx == n) ? (int64_t)idx[b] : (int64_t)(idx[b] / n) * ldx + (idx[b] % n);
          if (xf32) store4(xf + xo, mnew); else store4(xh + xo, mnew);
        }
      }
    }
  } else {
    for (int i = threadIdx.x; i < count; i += kEwThreads) {
      const int id = base + i;
      const float gv = load1(g + id);
      float mnew;
      if constexpr (MODE == MODE_TWO_BUFFER) {
        float a = load1(ac + id);
        mnew = mona_element(gv, load1(gp + id), a, mo[id], c);
        store1(gp + id, gv);
        store1(ac + id, a);
      } else if constexpr (MODE == MODE_ONE_BUFFER) {
        float cb = load1(ac + id);
        mnew = mona_element_one_buffer(gv, cb, mo[id], c);
        store1(ac + id, cb);
      } else {
        mnew = c.mu * mo[id] + gv;
      }
      ss += (double)mnew * mnew;
      mo[id] = mnew;
      const int64_t xo = (int64_t)(id / n) * ldx + (id % n);
      if (xf32) xf[xo] = mnew; else xh[xo] = (bf16_t)mnew;
    }
  }
  const double t = block_sum(ss, red);
  if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

// ||M||_F per matrix from the per-block partial sums, added in a fixed order in fp64 so the
// result does not depend on scheduling.  One wavefront per matrix.
//
// The products that follow accumulate the unscaled working copy in fp32 and apply 1 / ||M||_F^2 afterwards,
// which is exact only while the squares stay inside the fp32 range.  A norm outside [2^-40, 2^40] therefore
// sets MONA_STATUS_RESCALED: rescue_kernel then rewrites that matrix's working copy as M 2^e with
// ||M 2^e||_F in [1, 2), and the scale stored here is the one that belongs to the rewritten copy (a power
// of two moves no bit of any product, so the result is the one an unlimited exponent range would give).
constexpr double kNormLo = 9.094947017729282e-13;   // 2^-40
constexpr double kNormHi = 1099511627776.0;         // 2^40
__global__ __launch_bounds__(64) void norm_finalize_kernel(const MatStatic* __restrict__ stat,
                                                           const double* __restrict__ partials,
                                                           MatScale* __restrict__ scales,
                                                           const int32_t* __restrict__ list, float eps) {
  const int mat = list ? list[blockIdx.x] : blockIdx.x;
  const int first = stat[mat].first_block, nb = stat[mat].num_blocks;
  double s = 0.0;
  for (int i = threadIdx.x; i < nb; i += 64) s += partials[first + i];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  if (threadIdx.x == 0) {
    const double norm = sqrt(s);
    const double den = norm + (double)eps;
    MatScale r;
    r.norm = (float)fmin(norm, 3.402823466e38);
    r.status = 0u;
    r.xexp = 0;
    const bool finite = (s == s) && (s <= 1.7e308);
    if (!finite) {
      r.norm = (float)norm;
      r.inv = 0.0f;
      r.status = 2u;
    } else if (den <= 0.0) {
      r.inv = 0.0f;
      r.status = 1u;
    } else if (norm == 0.0 || (norm >= kNormLo && norm <= kNormHi)) {
      r.inv = 1.0f / ((float)norm + eps);
    } else {
      r.xexp = -ilogb(norm);
      r.inv = (float)ldexp(1.0 / den, -r.xexp);
      r.status = 4u;
    }
    r.inv2 = r.inv * r.inv;
    scales[mat] = r;
  }
}

// Repairs the working copies of the (rare) matrices norm_finalize_kernel has flagged, before any product
// reads them: a matrix with a non-finite norm gets an all-zero copy (its products then stay zero, so no
// NaN ever reaches the zero padding the Gram matrices rely on; its parameter is left alone anyway), and a
// matrix whose norm lies outside the safe window gets the copy M 2^e.  Every block scans the flags and
// leaves at once when none is set.
__global__ __launch_bounds__(256) void rescue_kernel(const MatStatic* __restrict__ stat,
                                                     const MatScale* __restrict__ scales,
                                                     const int32_t* __restrict__ list, int count) {
  int any = 0;
  for (int i = threadIdx.x; i < count; i += 256) any |= (scales[list ? list[i] : i].status & 6u) != 0;
  if (!__syncthreads_or(any)) return;
  for (int li = 0; li < count; ++li) {
    const int mat = list ? list[li] : li;
    const uint32_t st = scales[mat].status;
    if (!(st & 6u)) continue;
    const MatStatic ms = stat[mat];
    const int e = scales[mat].xexp;
    const int64_t total = (int64_t)ms.m * ms.n;
    bf16_t* __restrict__ xh = static_cast<bf16_t*>(ms.x);
    float* __restrict__ xf = static_cast<float*>(ms.x);
    for (int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x; id < total; id += (int64_t)gridDim.x * 256) {
      const int64_t xo = (id / ms.n) * ms.ldx + (id % ms.n);
      const float v = (st & 2u) ? 0.0f : ldexpf(ms.mom[id], e);
      if (ms.x_f32) xf[xo] = v; else xh[xo] = (bf16_t)v;
    }
  }
}

// Tables of a state that holds ONE matrix, written on the device from kernel arguments (for the entry
// point that may neither allocate nor copy from host memory).
__global__ __launch_bounds__(256) void single_tables_kernel(MatStatic ms, MatDynamic md, void* o_ptr, MatStatic* stat,
                                                            MatDynamic* dyn, void** o_ptrs, BlockWork* work,
                                                            int num_blocks, int32_t* members, int32_t* order) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i == 0) { stat[0] = ms; dyn[0] = md; o_ptrs[0] = o_ptr; members[0] = 0; order[0] = 0; }
  for (int b = i; b < num_blocks; b += gridDim.x * 256) work[b] = BlockWork{0, b};
}

// O = X_0 and the parameter update when no Newton-Schulz iteration is requested (T = 0),
// W <- (1 - eta lambda) W - eta gamma O   (Eq. muon_update).
template <typename WT>
__global__ __launch_bounds__(kEwThreads) void plain_update_kernel(
    const MatStatic* __restrict__ stat, const MatDynamic* __restrict__ dyn,
    const MatScale* __restrict__ scales, const BlockWork* __restrict__ work,
    void* const* __restrict__ o_ptrs, float lr, float wd, float gamma_coeff, int store_o, int want_w_dtype) {
  const BlockWork bw = work[blockIdx.x];
  const MatStatic ms = stat[bw.mat];
  if (ms.w_dtype != want_w_dtype) return;
  const MatScale sc = scales[bw.mat];
  if (sc.status & 2u) return;
  WT* __restrict__ w = static_cast<WT*>(dyn[bw.mat].w);
  const bool xf32 = ms.x_f32 != 0;
  const bf16_t* __restrict__ xh = static_cast<const bf16_t*>(ms.x);
  const float* __restrict__ xf = static_cast<const float*>(ms.x);
  bf16_t* __restrict__ oh = static_cast<bf16_t*>(o_ptrs[bw.mat]);
  float* __restrict__ of = static_cast<float*>(o_ptrs[bw.mat]);
  const int total = ms.m * ms.n;
  const int base = bw.chunk * kEwChunk;
  const int count = min(kEwChunk, total - base);
  const float gamma = gamma_coeff * sqrtf((float)max(ms.m, ms.n));
  const float keep = 1.0f - lr * wd, os = lr * gamma;
  for (int i = threadIdx.x; i < count; i += kEwThreads) {
    const int id = base + i;
    const int64_t xo = (int64_t)(id / ms.n) * ms.ldx + (id % ms.n);
    // O = X_0 in the working precision of this matrix
    const float ov = xf32 ? sc.inv * xf[xo] : stored<bf16_t>(sc.inv * (float)xh[xo]);
    if (store_o) {
      if (xf32) of[xo] = ov; else oh[xo] = (bf16_t)ov;
    }
    store1(w + id, keep * load1(w + id) - os * ov);
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* __restrict__ p, size_t n16) {
  const uint4 z = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    p[i] = z;
}

template <typename GT, typename ST, int MODE>
hipError_t launch_su(const MatStatic* stat, const MatDynamic* dyn, const BlockWork* work, double* partials,
                     int num_blocks, Coef c, hipStream_t s) {
  hipLaunchKernelGGL((state_update_kernel<GT, ST, MODE>), dim3(num_blocks), dim3(kEwThreads), 0, s, stat, dyn,
                     work, partials, c);
  return hipGetLastError();
}
template <int MODE>
hipError_t launch_su_mode(const MatStatic* stat, const MatDynamic* dyn, const BlockWork* work, double* partials,
                          int num_blocks, int g_bf16, int state_bf16, Coef c, hipStream_t s) {
  switch ((g_bf16 ? 2 : 0) | (state_bf16 ? 1 : 0)) {
    case 0: return launch_su<float, float, MODE>(stat, dyn, work, partials, num_blocks, c, s);
    case 1: return launch_su<float, bf16_t, MODE>(stat, dyn, work, partials, num_blocks, c, s);
    case 2: return launch_su<bf16_t, float, MODE>(stat, dyn, work, partials, num_blocks, c, s);
    default: return launch_su<bf16_t, bf16_t, MODE>(stat, dyn, work, partials, num_blocks, c, s);
  }
}

}  // namespace

// The gradient dtype may differ between matrices: the host orders the work table by gradient
// dtype and launches each dtype's range of blocks separately.
hipError_t launch_state_update(const MatStatic* stat, const MatDynamic* dyn, const BlockWork* work,
                               double* partials, int num_blocks, int g_bf16, int state_bf16, int one_buffer,
                               float mu, float beta_a, float alpha, int use_prev, hipStream_t s) {
  if (num_blocks <= 0) return hipSuccess;
  Coef c;
  c.mu = mu;
  c.beta = beta_a;
  c.one_minus_beta = 1.0f - beta_a;
  c.alpha = alpha;
  // use_prev: 0 = take D_k = 0 (first step with the first-difference flag), 1 = Alg. 1,
  //           2 = plain Muon (acceleration buffers untouched)
  c.use_prev = use_prev == 1;
  if (use_prev == 2) {
    // the state dtype does not matter: the acceleration buffers are not touched
    if (g_bf16) return launch_su<bf16_t, float, MODE_MUON>(stat, dyn, work, partials, num_blocks, c, s);
    return launch_su<float, float, MODE_MUON>(stat, dyn, work, partials, num_blocks, c, s);
  }
  if (one_buffer) return launch_su_mode<MODE_ONE_BUFFER>(stat, dyn, work, partials, num_blocks, g_bf16, state_bf16, c, s);
  return launch_su_mode<MODE_TWO_BUFFER>(stat, dyn, work, partials, num_blocks, g_bf16, state_bf16, c, s);
}

hipError_t launch_norm_finalize(const MatStatic* stat, const double* partials, MatScale* scales,
                                const int32_t* list, int count, float eps, hipStream_t s) {
  if (count <= 0) return hipSuccess;
  hipLaunchKernelGGL(norm_finalize_kernel, dim3(count), dim3(64), 0, s, stat, partials, scales, list, eps);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(rescue_kernel, dim3(1024), dim3(256), 0, s, stat, scales, list, count);
  return hipGetLastError();
}

hipError_t launch_single_tables(const MatStatic& ms, const MatDynamic& md, void* o_ptr, MatStatic* stat,
                                MatDynamic* dyn, void** o_ptrs, BlockWork* work, int num_blocks, int32_t* members,
                                int32_t* order, hipStream_t s) {
  const int blocks = num_blocks > 256 * 64 ? 64 : (num_blocks + 255) / 256;
  hipLaunchKernelGGL(single_tables_kernel, dim3(blocks > 0 ? blocks : 1), dim3(256), 0, s, ms, md, o_ptr, stat, dyn,
                     o_ptrs, work, num_blocks, members, order);
  return hipGetLastError();
}

hipError_t launch_plain_update(const MatStatic* stat, const MatDynamic* dyn, const MatScale* scales,
                               const BlockWork* work, int num_blocks, void* const* o_ptrs, float lr, float wd,
                               float gamma_coeff, int store_o, hipStream_t s) {
  if (num_blocks <= 0) return hipSuccess;
  // one launch per parameter dtype; blocks of the other dtype return at once
  hipLaunchKernelGGL((plain_update_kernel<float>), dim3(num_blocks), dim3(kEwThreads), 0, s, stat, dyn, scales,
                     work, o_ptrs, lr, wd, gamma_coeff, store_o, 0);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((plain_update_kernel<bf16_t>), dim3(num_blocks), dim3(kEwThreads), 0, s, stat, dyn, scales,
                     work, o_ptrs, lr, wd, gamma_coeff, store_o, 1);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  const size_t n16 = bytes / 16;   // the arena is carved in multiples of 256 bytes
  const int blocks = (int)((n16 + 255) / 256 < 8192 ? (n16 + 255) / 256 : 8192);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, s, static_cast<uint4*>(p), n16);
  return hipGetLastError();
}

}  // namespace mona
