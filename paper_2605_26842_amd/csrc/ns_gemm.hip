// Matrix products of the Newton-Schulz iteration (Eq. newton_schulz), written as three
// products per iteration on the short side p = min(m, n) of each matrix:
//
//     S   = X X^T                (p x p, symmetric)          "Gram"
//     B   = b S + c S S          (p x p, symmetric)          "poly"
//     X'  = a X + B X            (p x q)                     "apply"
//
// (for a tall matrix stored m x n with m > n the same polynomial is S = X^T X,
// X' = a X + X B, because the quintic is odd).  Every product has the form
//
//     out = post * (beta * E + alpha * P Q^T),     P: M x K,  Q: N x K
//
// over a batch of same-shape matrices.  An operand may be stored K-major (K x M); it is then
// transposed in registers on its way into LDS, so the MFMA loop below always reads K-contiguous
// rows.  All dimensions are padded by the host to multiples of the tile and the padding is kept
// zero, so the main loop has no bounds checks.
//
// bf16 path: v_mfma_f32_32x32x16_bf16, fp32 accumulation, 256 threads = 4 wavefronts in a
// 2 x 2 arrangement, block tile BM x BN (256 x 256 or 128 x 128), K step 64, LDS double buffer.
// fp32 path: v_mfma_f32_32x32x2_f32, 128 x 128 tiles, K step 16.
#include "mona_internal.h"

#include <cstdlib>

namespace mona {

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kXcds = 8;   // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

// compile-time loop: f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>)
template <int I> struct IC { static constexpr int value = I; constexpr operator int() const { return I; } };
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(IC<I>{});
    static_for<N, I + 1>(f);
  }
}

// ---- tile decode ---------------------------------------------------------------------
struct TileId {
  int mat, ti, tj;
  bool valid;
};

// Workgroup L runs on die L % 8.  Give every die one contiguous range of the logical tile
// order (matrix-major), so that tiles that share operands share that die's L2.
__device__ __forceinline__ TileId decode_tile(const GemmArgs& a) {
  TileId t;
  const int total = a.tiles_per_mat * a.count;
  const int per_xcd = gridDim.x / kXcds;
  const int logical = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
  t.valid = logical < total;
  t.mat = logical / a.tiles_per_mat;
  int r = logical - t.mat * a.tiles_per_mat;
  if (a.symmetric) {
    int ti = 0, row = a.tiles_n;
    while (r >= row) { r -= row; --row; ++ti; }
    t.ti = ti;
    t.tj = ti + r;
  } else {
    t.ti = r / a.tiles_n;
    t.tj = r - t.ti * a.tiles_n;
  }
  return t;
}

// ---- LDS layout ------------------------------------------------------------------------
// An operand tile is R rows of 64 bf16 (128 bytes = 8 chunks of 16 bytes).  The chunk index is
// XOR-swizzled with the row so that 16 consecutive rows at one logical chunk fall on 16
// different 16-byte bank groups (the fragment read), as do 2 rows x 8 chunks (the tile store).
__device__ __forceinline__ int lds_slot(int row, int chunk) {
  return row * 8 + (chunk ^ ((row & 7) ^ ((row >> 3) & 1)));
}

__device__ __forceinline__ uint32_t pack_lo(uint32_t x, uint32_t y) {  // (x.lo16, y.lo16)
  return __builtin_amdgcn_perm(y, x, 0x05040100u);
}
__device__ __forceinline__ uint32_t pack_hi(uint32_t x, uint32_t y) {  // (x.hi16, y.hi16)
  return __builtin_amdgcn_perm(y, x, 0x07060302u);
}

// ---- operand loaders (global -> registers -> LDS) ---------------------------------------
// R: rows of the tile (BM or BN).  Each thread moves R/32 chunks of 16 bytes per K step.
template <int R, bool TRANS>
struct Loader {
  static constexpr int kRegs = R / 32;
  u32x4 v[kRegs];

  // src: first element of this matrix; r0: first tile row; k0: first k; ld: leading dimension
  __device__ __forceinline__ void load(const bf16_t* __restrict__ src, int ld, int r0, int k0) {
    const int tid = threadIdx.x;
    if constexpr (!TRANS) {
      const int chunk = tid & 7, row = tid >> 3;
      static_for<kRegs>([&](auto i) {
        v[i] = *reinterpret_cast<const u32x4*>(src + (size_t)(r0 + row + 32 * i) * ld + k0 + chunk * 8);
      });
    } else {
      // K-major storage: element (k, r) at src[k * ld + r].  Each thread takes kRegs consecutive
      // k-rows of 8 consecutive r.
      constexpr int kKB = 64 / kRegs;           // k-blocks per K step
      const int kb = tid % kKB, rb = tid / kKB;
      static_for<kRegs>([&](auto i) {
        v[i] = *reinterpret_cast<const u32x4*>(src + (size_t)(k0 + kb * kRegs + i) * ld + r0 + rb * 8);
      });
    }
  }

  __device__ __forceinline__ void store(u32x4* __restrict__ lds) const {
    const int tid = threadIdx.x;
    if constexpr (!TRANS) {
      const int chunk = tid & 7, row = tid >> 3;
      static_for<kRegs>([&](auto i) { lds[lds_slot(row + 32 * i, chunk)] = v[i]; });
    } else {
      constexpr int kKB = 64 / kRegs;
      const int kb = tid % kKB, rb = tid / kKB;
      // transpose the kRegs x 8 block held in v[] to 8 rows of kRegs k-values
      // word(i, cw): 32-bit word cw of k-row i, i.e. columns 2 cw and 2 cw + 1
      auto word = [&](int i, int cw) -> uint32_t {
        return cw == 0 ? v[i].x : cw == 1 ? v[i].y : cw == 2 ? v[i].z : v[i].w;
      };
      if constexpr (kRegs == 8) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          u32x4 o;
          const int cw = c >> 1;
          if ((c & 1) == 0) {
            o.x = pack_lo(word(0, cw), word(1, cw));
            o.y = pack_lo(word(2, cw), word(3, cw));
            o.z = pack_lo(word(4, cw), word(5, cw));
            o.w = pack_lo(word(6, cw), word(7, cw));
          } else {
            o.x = pack_hi(word(0, cw), word(1, cw));
            o.y = pack_hi(word(2, cw), word(3, cw));
            o.z = pack_hi(word(4, cw), word(5, cw));
            o.w = pack_hi(word(6, cw), word(7, cw));
          }
          lds[lds_slot(rb * 8 + c, kb)] = o;
        }
      } else {
        static_assert(kRegs == 4 || kRegs == 8, "tile rows must be 128 or 256");
        // 4 k-values per row: half a chunk
        u32x2* lds2 = reinterpret_cast<u32x2*>(lds);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          u32x2 o;
          const int cw = c >> 1;
          if ((c & 1) == 0) {
            o.x = pack_lo(word(0, cw), word(1, cw));
            o.y = pack_lo(word(2, cw), word(3, cw));
          } else {
            o.x = pack_hi(word(0, cw), word(1, cw));
            o.y = pack_hi(word(2, cw), word(3, cw));
          }
          lds2[lds_slot(rb * 8 + c, kb >> 1) * 2 + (kb & 1)] = o;
        }
      }
    }
  }
};

__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
__device__ __forceinline__ float to_f32(float v) { return v; }

// ---- epilogue -----------------------------------------------------------------------------
// The accumulators of a wavefront (MI x NI blocks of 32 x 32; acc[v] of a block sits at
// row = (v / 4) * 8 + (lane / 32) * 4 + (v % 4), col = lane % 32) are staged through LDS one
// 32-row band at a time, so that every global access of the epilogue is a 16-byte vector that
// runs along a row:  out = post * (beta * E + alpha * acc), then either a plain store (plus the
// mirrored store of a symmetric product) or the parameter update of Eq. muon_update.
template <typename T> struct Chunk;           // 16 bytes of T
template <> struct Chunk<bf16_t> { static constexpr int N = 8; typedef bf16x8 vec; };
template <> struct Chunk<float> { static constexpr int N = 4; typedef f32x4 vec; };

template <typename T, int WN, int MI, int NI>
__device__ __forceinline__ void tile_epilogue(const GemmArgs& a, f32x16 (&acc)[MI][NI], float* __restrict__ lds_f,
                                              int tmat, int row_w0, int col_w0, bool mirror) {
  constexpr int CH = Chunk<T>::N;
  typedef typename Chunk<T>::vec vec_t;
  constexpr int LDW = WN + 4;                    // floats per staged row (+4: the two half-waves
                                                 // write rows 4 apart, keep them on different banks)
  constexpr int CPR = WN / CH;                   // chunks per row
  constexpr int PASSES = 32 * CPR / 64;          // chunks per lane per band
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* __restrict__ stage = lds_f + wave * (32 * LDW);

  const int mi = a.members ? a.members[tmat] : tmat;
  float post = 1.0f;
  if (a.post == POST_INV) post = a.scales[mi].inv;
  else if (a.post == POST_INV2) post = a.scales[mi].inv2;
  const T* __restrict__ E = a.E ? static_cast<const T*>(a.E) + (size_t)tmat * a.strideE : nullptr;
  T* __restrict__ C = static_cast<T*>(a.C) + (size_t)tmat * a.strideC;
  const bool update = a.epilogue == EPI_UPDATE;
  int wm_real = 0, wn_real = 0, w_is_bf16 = 0;
  bool skip_w = true;
  void* wptr = nullptr;
  if (update) {
    const MatStatic& ms = a.stat[mi];
    wm_real = ms.m; wn_real = ms.n; w_is_bf16 = ms.w_dtype;
    wptr = a.dyn[mi].w;
    skip_w = (a.scales[mi].status & 2u) != 0;
  }
  const bool w_vec_ok = (wn_real % CH) == 0;

  static_for<MI>([&](auto i) {
    // the band's E operands are fetched up front: their latency overlaps the staging below
    vec_t ev[PASSES];
    if (E != nullptr) {
#pragma unroll
      for (int pss = 0; pss < PASSES; ++pss) {
        const int idx = pss * 64 + lane;
        ev[pss] = *reinterpret_cast<const vec_t*>(E + (size_t)(row_w0 + i * 32 + idx / CPR) * a.lde + col_w0 +
                                                  (idx % CPR) * CH);
      }
    }
    __syncthreads();     // previous band fully consumed (first band: operand tiles no longer read)
    static_for<NI>([&](auto j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        stage[r * LDW + j * 32 + (lane & 31)] = acc[i][j][v];
      }
    });
    __syncthreads();
#pragma unroll
    for (int pss = 0; pss < PASSES; ++pss) {
      const int idx = pss * 64 + lane;
      const int r = idx / CPR, ch = idx % CPR;
      const int grow = row_w0 + i * 32 + r, gcol = col_w0 + ch * CH;
      float val[CH];
      {
        const f32x4* src = reinterpret_cast<const f32x4*>(stage + r * LDW + ch * CH);
#pragma unroll
        for (int q = 0; q < CH / 4; ++q) {
          const f32x4 t4 = src[q];
          val[q * 4 + 0] = t4.x; val[q * 4 + 1] = t4.y; val[q * 4 + 2] = t4.z; val[q * 4 + 3] = t4.w;
        }
      }
      if (E != nullptr) {
#pragma unroll
        for (int e = 0; e < CH; ++e) val[e] = post * (a.alpha * val[e] + a.beta * to_f32(ev[pss][e]));
      } else {
#pragma unroll
        for (int e = 0; e < CH; ++e) val[e] = post * (a.alpha * val[e]);
      }
      vec_t ov;
#pragma unroll
      for (int e = 0; e < CH; ++e) ov[e] = (T)val[e];
      if (!update || a.store_out) *reinterpret_cast<vec_t*>(C + (size_t)grow * a.ldc + gcol) = ov;
      if (mirror) {
        // keep the rounded result for the transposed store below
        f32x4* dst = reinterpret_cast<f32x4*>(stage + r * LDW + ch * CH);
#pragma unroll
        for (int q = 0; q < CH / 4; ++q) {
          f32x4 t4 = {to_f32(ov[q * 4 + 0]), to_f32(ov[q * 4 + 1]), to_f32(ov[q * 4 + 2]), to_f32(ov[q * 4 + 3])};
          dst[q] = t4;
        }
      }
      if (update && !skip_w && grow < wm_real) {
        // W <- (1 - eta lambda) W - eta gamma O, O as stored in the working precision
        const size_t wi = (size_t)grow * wn_real + gcol;
        if (w_vec_ok && gcol + CH <= wn_real) {
          if (w_is_bf16) {
            typedef bf16_t wv_t __attribute__((ext_vector_type(CH)));
            wv_t* wp = reinterpret_cast<wv_t*>(static_cast<bf16_t*>(wptr) + wi);
            wv_t wv = *wp;
#pragma unroll
            for (int e = 0; e < CH; ++e) wv[e] = (bf16_t)(a.w_keep * (float)wv[e] - a.o_scale * to_f32(ov[e]));
            *wp = wv;
          } else {
            f32x4* wp = reinterpret_cast<f32x4*>(static_cast<float*>(wptr) + wi);
#pragma unroll
            for (int q = 0; q < CH / 4; ++q) {
              f32x4 wv = wp[q];
#pragma unroll
              for (int e = 0; e < 4; ++e) wv[e] = a.w_keep * wv[e] - a.o_scale * to_f32(ov[q * 4 + e]);
              wp[q] = wv;
            }
          }
        } else {
#pragma unroll
          for (int e = 0; e < CH; ++e) {
            if (gcol + e < wn_real) {
              if (w_is_bf16) {
                bf16_t* w = static_cast<bf16_t*>(wptr) + wi + e;
                *w = (bf16_t)(a.w_keep * (float)*w - a.o_scale * to_f32(ov[e]));
              } else {
                float* w = static_cast<float*>(wptr) + wi + e;
                *w = a.w_keep * *w - a.o_scale * to_f32(ov[e]);
              }
            }
          }
        }
      }
    }
    if (mirror) {
      // transposed copy of this band: C[col][row], 16-byte pieces along the band's 32 rows
      __syncthreads();
      constexpr int RCH = 32 / CH;               // row-chunks per band
      constexpr int MPASSES = WN * RCH / 64;
#pragma unroll
      for (int pss = 0; pss < MPASSES; ++pss) {
        const int idx = pss * 64 + lane;
        const int c = idx % WN, rc = idx / WN;
        vec_t ov;
#pragma unroll
        for (int e = 0; e < CH; ++e) ov[e] = (T)stage[(rc * CH + e) * LDW + c];
        *reinterpret_cast<vec_t*>(C + (size_t)(col_w0 + c) * a.ldc + row_w0 + i * 32 + rc * CH) = ov;
      }
    }
  });
}

// ---- bf16 kernel -----------------------------------------------------------------------------
template <int BM, int BN, bool TP, bool TQ>
__global__ __launch_bounds__(kThreads) void ns_gemm_bf16_kernel(const GemmArgs a) {
  constexpr int BK = 64;
  constexpr int WM = BM / 2, WN = BN / 2;   // per-wavefront tile
  constexpr int MI = WM / 32, NI = WN / 32; // MFMA blocks per wavefront
  __shared__ __attribute__((aligned(16))) u32x4 lds[2][(BM + BN) * 8];

  const TileId t = decode_tile(a);
  if (!t.valid) return;

  const bf16_t* __restrict__ P = static_cast<const bf16_t*>(a.P) + (size_t)t.mat * a.strideP;
  const bf16_t* __restrict__ Q = static_cast<const bf16_t*>(a.Q) + (size_t)t.mat * a.strideQ;
  const int m0 = t.ti * BM, n0 = t.tj * BN;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  Loader<BM, TP> lp;
  Loader<BN, TQ> lq;
  const int KT = a.K / BK;

  // Software pipeline: tile kt+1 travels global -> registers while tile kt is multiplied, and is
  // written to the other LDS buffer during the last quarter of the step; MFMA fragments are
  // double-buffered so the reads of quarter kk+1 are in flight while quarter kk is multiplied.
  const int frow = lane & 31, fchunk = lane >> 5;
  bf16x8 fa[2][MI], fb[2][NI];
  auto load_frags = [&](auto slot, int buf, int kk) {
    const u32x4* __restrict__ ps = lds[buf];
    const u32x4* __restrict__ qs = lds[buf] + BM * 8;
    static_for<MI>([&](auto i) {
      fa[slot][i] = __builtin_bit_cast(bf16x8, ps[lds_slot(wm * WM + i * 32 + frow, kk * 2 + fchunk)]);
    });
    static_for<NI>([&](auto j) {
      fb[slot][j] = __builtin_bit_cast(bf16x8, qs[lds_slot(wn * WN + j * 32 + frow, kk * 2 + fchunk)]);
    });
  };
  auto multiply = [&](auto slot) {
    static_for<MI>([&](auto i) {
      static_for<NI>([&](auto j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
      });
    });
  };
  auto kstep = [&](auto has_next, int kt) {
    const int buf = kt & 1;
    if constexpr (has_next) {
      lp.load(P, a.ldp, m0, (kt + 1) * BK);
      lq.load(Q, a.ldq, n0, (kt + 1) * BK);
    }
    // keep the phases of the step in program order: the loads above must be issued a full step
    // before their data is needed, not sunk next to the LDS writes that consume them
    __builtin_amdgcn_sched_barrier(0);
    static_for<BK / 16>([&](auto kk) {
      if constexpr (kk + 1 < BK / 16) load_frags(IC<(kk + 1) & 1>{}, buf, kk + 1);
      if constexpr (has_next && kk == BK / 16 - 1) {
        lp.store(lds[buf ^ 1]);
        lq.store(lds[buf ^ 1] + BM * 8);
      }
      multiply(IC<kk & 1>{});
      __builtin_amdgcn_sched_barrier(0);
    });
    __syncthreads();
    if constexpr (has_next) load_frags(IC<0>{}, buf ^ 1, 0);
  };

  lp.load(P, a.ldp, m0, 0);
  lq.load(Q, a.ldq, n0, 0);
  lp.store(lds[0]);
  lq.store(lds[0] + BM * 8);
  __syncthreads();
  load_frags(IC<0>{}, 0, 0);
  for (int kt = 0; kt + 1 < KT; ++kt) kstep(IC<1>{}, kt);
  kstep(IC<0>{}, KT - 1);

  const bool mirror = a.symmetric && (t.ti != t.tj);
  tile_epilogue<bf16_t, WN, MI, NI>(a, acc, reinterpret_cast<float*>(&lds[0][0]), t.mat, m0 + wm * WM, n0 + wn * WN,
                                    mirror);
}

// ---- bf16 kernel, direct-to-LDS pipeline ------------------------------------------------------
// 256 x 256 tile, 512 threads = 8 wavefronts (2 x 4, each 128 x 64), two per SIMD so that one
// multiplies while the other waits on LDS.  Operand tiles go from global memory straight into
// LDS (global_load_lds, 16 bytes per lane, no staging registers) through a ring of 4 stages of
// K = 32, so a tile is requested three steps (~3000 MFMA cycles per SIMD) before it is used.
//
// LDS layouts of one 256 x 32 operand tile (16 KB), in 16-byte chunks:
//   row-major operand (K contiguous in memory): 256 rows x 4 chunks, chunk c of row r at
//     r * 4 + (c ^ ((r >> 2) & 3)); a fragment is one ds_read_b128 per lane (8 consecutive k);
//   K-major operand (stored K x M): 32 k-rows x 32 chunks, chunk c of k-row k at
//     k * 32 + (c ^ ((k & 3) << 2)); a fragment is two ds_read_b64_tr_b16 per lane: 16 lanes
//     fetch a 4 (k) x 16 (m) block and each receives the 4 k-values of one m.
// A direct load writes lane l's 16 bytes at (wave-uniform base) + 16 l, so the swizzle is applied
// by choosing which global chunk each lane fetches.
constexpr int kThreadsV2 = 512;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
#define MONA_AS1 __attribute__((address_space(1)))
#define MONA_AS3 __attribute__((address_space(3)))

template <bool TP, bool TQ>
__global__ __launch_bounds__(kThreadsV2) void ns_gemm_bf16_v2_kernel(const GemmArgs a) {
  constexpr int BM = 256, BN = 256, BK = 32, STAGES = 4;
  constexpr int WM = 128, WN = 64, MI = 4, NI = 2;
  constexpr int TILE_U = 1024;                 // 16-byte units per operand tile
  constexpr int STAGE_U = 2 * TILE_U;          // P tile then Q tile
  __shared__ __attribute__((aligned(16))) u32x4 lds[STAGES * STAGE_U];   // 128 KB

  const TileId t = decode_tile(a);
  if (!t.valid) return;
  const bf16_t* __restrict__ P = static_cast<const bf16_t*>(a.P) + (size_t)t.mat * a.strideP;
  const bf16_t* __restrict__ Q = static_cast<const bf16_t*>(a.Q) + (size_t)t.mat * a.strideQ;
  const int m0 = t.ti * BM, n0 = t.tj * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3;

  // ---- direct loads: 2 instructions per wavefront per operand per stage ----
  const bf16_t* gp[2];
  const bf16_t* gq[2];
  static_for<2>([&](auto q) {
    const int S = (wave * 2 + q) * 64 + lane;
    if constexpr (!TP) {
      const int row = S >> 2, c = (S & 3) ^ ((row >> 2) & 3);
      gp[q] = P + (size_t)(m0 + row) * a.ldp + c * 8;
    } else {
      const int k = S >> 5, c = (S & 31) ^ ((k & 3) << 2);
      gp[q] = P + (size_t)k * a.ldp + m0 + c * 8;
    }
    if constexpr (!TQ) {
      const int row = S >> 2, c = (S & 3) ^ ((row >> 2) & 3);
      gq[q] = Q + (size_t)(n0 + row) * a.ldq + c * 8;
    } else {
      const int k = S >> 5, c = (S & 31) ^ ((k & 3) << 2);
      gq[q] = Q + (size_t)k * a.ldq + n0 + c * 8;
    }
  });
  const size_t incp = TP ? (size_t)BK * a.ldp : (size_t)BK;   // elements per K step
  const size_t incq = TQ ? (size_t)BK * a.ldq : (size_t)BK;
  auto issue = [&](auto stage, int kt) {
    static_for<2>([&](auto q) {
      u32x4* dp = lds + stage * STAGE_U + (wave * 2 + q) * 64;
      u32x4* dq = dp + TILE_U;
      __builtin_amdgcn_global_load_lds((const MONA_AS1 void*)(gp[q] + kt * incp), (MONA_AS3 void*)dp, 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const MONA_AS1 void*)(gq[q] + kt * incq), (MONA_AS3 void*)dq, 16, 0, 0);
    });
  };

  // ---- fragment addresses (bytes inside an operand tile), per lane ----
  // row-major layout: two variants of the chunk term, one per 16-wide k step
  const int rsw = ((lane & 31) >> 2) & 3;                 // (row >> 2) & 3, the same for every block
  const int r_off[2] = {((lane & 31) * 4 + (((0 + (lane >> 5)) ^ rsw))) * 16,
                        ((lane & 31) * 4 + (((2 + (lane >> 5)) ^ rsw))) * 16};
  // K-major layout: k-row and 16-byte chunk this lane fetches for a 4 x 16 transposed block
  const int t_k = 8 * (lane >> 5) + ((lane & 15) >> 2);    // + 16 kk + 4 quad
  const int t_x = (lane & 15) >> 2;                        // k & 3 of that row: the swizzle term
  const int t_nl = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);  // m inside the 32-wide block
  int ta_off[MI], tb_off[NI];
  static_for<MI>([&](auto i) {
    const int c = (wm * (WM / 8) + i * 4 + (t_nl >> 3)) ^ (t_x << 2);
    ta_off[i] = t_k * 512 + c * 16 + (t_nl & 7) * 2;
  });
  static_for<NI>([&](auto j) {
    const int c = (wn * (WN / 8) + j * 4 + (t_nl >> 3)) ^ (t_x << 2);
    tb_off[j] = t_k * 512 + c * 16 + (t_nl & 7) * 2;
  });

  f32x16 acc[MI][NI];
  static_for<MI>([&](auto i) {
    static_for<NI>([&](auto j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    });
  });

  auto frag_r = [&](const char* tile, int blk_row, auto kk) -> bf16x8 {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(tile + blk_row * 64 + r_off[kk]));
  };
  // Transposed fragments are read with inline assembly: the compiler cannot tell that these LDS
  // reads do not touch the stages still being filled by direct loads and would wait for all of
  // those first.  The reads return through the LGKM counter; wait_frags() below waits for it.
  auto frag_t = [&](uint32_t tile_addr, int off, auto kk, u32x2& lo, u32x2& hi) {
    const uint32_t p0 = tile_addr + off + kk * (16 * 512);
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(p0));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:2048" : "=v"(hi) : "v"(p0));
  };
  auto compute = [&](auto stage) {
    const char* tp = reinterpret_cast<const char*>(lds + stage * STAGE_U);
    const char* tq = tp + TILE_U * 16;
    const uint32_t tp_addr = (uint32_t)(uintptr_t)(MONA_AS3 const char*)tp;
    const uint32_t tq_addr = tp_addr + TILE_U * 16;
    static_for<BK / 16>([&](auto kk) {
      bf16x8 fa[MI], fb[NI];
      u32x2 ta[MI][2], tb[NI][2];
      static_for<MI>([&](auto i) {
        if constexpr (!TP) fa[i] = frag_r(tp, wm * WM + i * 32, kk);
        else frag_t(tp_addr, ta_off[i], kk, ta[i][0], ta[i][1]);
      });
      static_for<NI>([&](auto j) {
        if constexpr (!TQ) fb[j] = frag_r(tq, wn * WN + j * 32, kk);
        else frag_t(tq_addr, tb_off[j], kk, tb[j][0], tb[j][1]);
      });
      if constexpr (TP) {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(ta[0][0]), "+v"(ta[0][1]), "+v"(ta[1][0]), "+v"(ta[1][1]), "+v"(ta[2][0]), "+v"(ta[2][1]),
                       "+v"(ta[3][0]), "+v"(ta[3][1]));
        static_for<MI>([&](auto i) {
          const u32x4 v = {ta[i][0].x, ta[i][0].y, ta[i][1].x, ta[i][1].y};
          fa[i] = __builtin_bit_cast(bf16x8, v);
        });
      }
      if constexpr (TQ) {
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(tb[0][0]), "+v"(tb[0][1]), "+v"(tb[1][0]), "+v"(tb[1][1]));
        static_for<NI>([&](auto j) {
          const u32x4 v = {tb[j][0].x, tb[j][0].y, tb[j][1].x, tb[j][1].y};
          fb[j] = __builtin_bit_cast(bf16x8, v);
        });
      }
      static_for<MI>([&](auto i) {
        static_for<NI>([&](auto j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        });
      });
    });
  };

  // s_waitcnt vmcnt(n), leaving the other counters alone (gfx9 encoding)
#define MONA_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

  const int KT = a.K / BK;      // a multiple of 4: K is a multiple of 128
  issue(IC<0>{}, 0);
  issue(IC<1>{}, 1);
  issue(IC<2>{}, 2);
  // each wavefront has 4 loads per stage in flight; stage kt is complete once at most 8 newer remain.
  // A bare s_barrier (no fence) is used inside the pipeline: a fence would drain every load in flight.
  int kt = 0;
  for (; kt + 4 < KT; kt += 4) {
    static_for<4>([&](auto u) {
      MONA_WAIT_VM(8);
      __builtin_amdgcn_s_barrier();        // stage kt landed for everyone, stage kt+3 free for everyone
      issue(IC<(u + 3) & 3>{}, kt + u + 3);
      compute(u);
    });
  }
  // last four steps: one more tile to request, then drain
  MONA_WAIT_VM(8);
  __builtin_amdgcn_s_barrier();
  issue(IC<3>{}, kt + 3);
  compute(IC<0>{});
  MONA_WAIT_VM(8);
  __builtin_amdgcn_s_barrier();
  compute(IC<1>{});
  MONA_WAIT_VM(4);
  __builtin_amdgcn_s_barrier();
  compute(IC<2>{});
  MONA_WAIT_VM(0);
  __builtin_amdgcn_s_barrier();
  compute(IC<3>{});
#undef MONA_WAIT_VM

  const bool mirror = a.symmetric && (t.ti != t.tj);
  tile_epilogue<bf16_t, WN, MI, NI>(a, acc, reinterpret_cast<float*>(&lds[0]), t.mat, m0 + wm * WM, n0 + wn * WN,
                                    mirror);
}

// ---- fp32 kernel ------------------------------------------------------------------------------
// 128 x 128 tile, K step 16.  LDS holds each operand k-major ([k][row], padded) so a fragment
// read (32 consecutive rows at one k) is conflict-free.
template <bool TP, bool TQ>
__global__ __launch_bounds__(kThreads) void ns_gemm_f32_kernel(const GemmArgs a) {
  constexpr int BM = 128, BN = 128, BK = 16;
  constexpr int LDR = 128 + 4;   // padded row count per k
  constexpr int kStageFloats = 4 * 32 * (64 + 4);          // epilogue staging, 4 wavefronts
  constexpr int kTileFloats = 2 * 2 * BK * LDR;
  __shared__ __attribute__((aligned(16))) float lds_raw[kTileFloats > kStageFloats ? kTileFloats : kStageFloats];
  float (*lds)[2][BK * LDR] = reinterpret_cast<float (*)[2][BK * LDR]>(lds_raw);

  const TileId t = decode_tile(a);
  if (!t.valid) return;
  const float* __restrict__ P = static_cast<const float*>(a.P) + (size_t)t.mat * a.strideP;
  const float* __restrict__ Q = static_cast<const float*>(a.Q) + (size_t)t.mat * a.strideQ;
  const int m0 = t.ti * BM, n0 = t.tj * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tid = threadIdx.x;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  // each thread moves 2 x float4 per operand per K step
  f32x4 rp[2], rq[2];
  auto gload = [&](const float* __restrict__ src, int ld, int r0, int k0, bool trans, f32x4* r) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + i * kThreads;               // 0..511 float4 slots of a 128 x 16 tile
      if (!trans) {
        const int row = id >> 2, kq = id & 3;          // 4 float4 per row (16 k)
        r[i] = *reinterpret_cast<const f32x4*>(src + (size_t)(r0 + row) * ld + k0 + kq * 4);
      } else {
        const int k = id >> 5, rq4 = id & 31;          // 32 float4 per k-row (128 rows)
        r[i] = *reinterpret_cast<const f32x4*>(src + (size_t)(k0 + k) * ld + r0 + rq4 * 4);
      }
    }
  };
  auto lstore = [&](float* __restrict__ dst, bool trans, const f32x4* r) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + i * kThreads;
      if (!trans) {
        const int row = id >> 2, kq = id & 3;
        dst[(kq * 4 + 0) * LDR + row] = r[i].x;
        dst[(kq * 4 + 1) * LDR + row] = r[i].y;
        dst[(kq * 4 + 2) * LDR + row] = r[i].z;
        dst[(kq * 4 + 3) * LDR + row] = r[i].w;
      } else {
        const int k = id >> 5, rq4 = id & 31;
        *reinterpret_cast<f32x4*>(dst + k * LDR + rq4 * 4) = r[i];
      }
    }
  };

  const int KT = a.K / BK;
  gload(P, a.ldp, m0, 0, TP, rp);
  gload(Q, a.ldq, n0, 0, TQ, rq);
  lstore(lds[0][0], TP, rp);
  lstore(lds[0][1], TQ, rq);
  __syncthreads();
  const int frow = lane & 31, fk = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) {
      gload(P, a.ldp, m0, (kt + 1) * BK, TP, rp);
      gload(Q, a.ldq, n0, (kt + 1) * BK, TQ, rq);
    }
    const float* __restrict__ sp = lds[buf][0];
    const float* __restrict__ sq = lds[buf][1];
#pragma unroll
    for (int kk = 0; kk < BK / 2; ++kk) {
      float fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = sp[(kk * 2 + fk) * LDR + wm * 64 + i * 32 + frow];
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = sq[(kk * 2 + fk) * LDR + wn * 64 + j * 32 + frow];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      lstore(lds[buf ^ 1][0], TP, rp);
      lstore(lds[buf ^ 1][1], TQ, rq);
    }
    __syncthreads();
  }

  const bool mirror = a.symmetric && (t.ti != t.tj);
  tile_epilogue<float, 64, 2, 2>(a, acc, lds_raw, t.mat, m0 + wm * 64, n0 + wn * 64, mirror);
}

template <int BM, int BN>
hipError_t launch_bf16(const GemmArgs& a, bool tp, bool tq, int grid, hipStream_t s) {
  if (!tp && !tq) hipLaunchKernelGGL((ns_gemm_bf16_kernel<BM, BN, false, false>), dim3(grid), dim3(kThreads), 0, s, a);
  else if (!tp && tq) hipLaunchKernelGGL((ns_gemm_bf16_kernel<BM, BN, false, true>), dim3(grid), dim3(kThreads), 0, s, a);
  else if (tp && tq) hipLaunchKernelGGL((ns_gemm_bf16_kernel<BM, BN, true, true>), dim3(grid), dim3(kThreads), 0, s, a);
  else return hipErrorInvalidValue;   // (transposed P, plain Q) never occurs in the plan
  return hipGetLastError();
}

}  // namespace

// development switch: MONA_GEMM_V1=1 selects the register-staged 256-tile kernel
static const bool g_use_v2 = []() { const char* e = getenv("MONA_GEMM_V1"); return !(e && e[0] == '1'); }();

hipError_t launch_ns_gemm(const GemmArgs& a, int tile, bool transP, bool transQ, bool f32, hipStream_t s) {
  const long long total = (long long)a.tiles_per_mat * a.count;
  if (total <= 0) return hipSuccess;
  if (total > 0x7fffff00LL) return hipErrorInvalidValue;
  const int grid = (int)((total + kXcds - 1) / kXcds) * kXcds;
  if (f32) {
    if (tile != 128) return hipErrorInvalidValue;
    if (!transP && !transQ) hipLaunchKernelGGL((ns_gemm_f32_kernel<false, false>), dim3(grid), dim3(kThreads), 0, s, a);
    else if (!transP && transQ) hipLaunchKernelGGL((ns_gemm_f32_kernel<false, true>), dim3(grid), dim3(kThreads), 0, s, a);
    else if (transP && transQ) hipLaunchKernelGGL((ns_gemm_f32_kernel<true, true>), dim3(grid), dim3(kThreads), 0, s, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
  }
  if (tile == 256 && g_use_v2) {
    if (!transP && !transQ) hipLaunchKernelGGL((ns_gemm_bf16_v2_kernel<false, false>), dim3(grid), dim3(kThreadsV2), 0, s, a);
    else if (!transP && transQ) hipLaunchKernelGGL((ns_gemm_bf16_v2_kernel<false, true>), dim3(grid), dim3(kThreadsV2), 0, s, a);
    else if (transP && transQ) hipLaunchKernelGGL((ns_gemm_bf16_v2_kernel<true, true>), dim3(grid), dim3(kThreadsV2), 0, s, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
  }
  if (tile == 256) return launch_bf16<256, 256>(a, transP, transQ, grid, s);
  if (tile == 128) return launch_bf16<128, 128>(a, transP, transQ, grid, s);
  return hipErrorInvalidValue;
}

}  // namespace mona
