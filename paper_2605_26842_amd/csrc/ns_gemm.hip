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
// over a batch of same-shape matrices.  An operand may be stored K-major (K x M).  All dimensions
// are padded by the host to multiples of the tile and the padding is kept zero, so the main loops
// have no bounds checks.  Symmetric products compute the block-upper-triangular tiles and mirror them.
//
// Three kernels:
//   ns_gemm_bf16_dma_kernel  the workhorse: persistent, 256 x 256 tile, 8 wavefronts of 128 x 64,
//                            v_mfma_f32_32x32x16_bf16 with fp32 accumulation, operands sent straight from
//                            global memory into a ring of four LDS stages of K = 32 (K-major tiles
//                            are read from LDS with the transposing read), epilogue BlockEpilogue;
//   ns_gemm_bf16_kernel      128 x 128 tile, 4 wavefronts, register-staged LDS double buffer of K = 64
//                            (a K-major operand is transposed in registers on its way into LDS), for
//                            launches too small to fill the chip with large tiles;
//   ns_gemm_f32_kernel       v_mfma_f32_32x32x2_f32, 128 x 128 tile, K step 16, for fp32 products.
#include "mona_internal.h"

#include <type_traits>

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
constexpr int kBandRows = 6;

struct TileId {
  int mat, ti, tj;
  bool valid;
};

// Workgroup L runs on die L % 8.  Give every die one contiguous range of the logical tile
// order (matrix-major), so that tiles that share operands share that die's L2.
__device__ __forceinline__ TileId decode_logical(const GemmArgs& a, int logical, bool in_range) {
  TileId t;
  const int total = a.tiles_per_mat * a.count;
  t.valid = in_range && logical < total;
  t.mat = logical / a.tiles_per_mat;
  int r = logical - t.mat * a.tiles_per_mat;
  if (a.symmetric) {
    // row block ti holds the column blocks from its diagonal onwards: tj >= ratio * ti,
    // ratio = tile rows / tile columns
    int ti = 0, row = a.tiles_n;
    while (r >= row && row > 0) { r -= row; row -= a.sym_ratio; ++ti; }
    t.ti = ti;
    t.tj = ti * a.sym_ratio + r;
  } else {
    // Bands of up to kBandRows tile rows, walked column by column: the 32 workgroups of a die then hold
    // a block of about 6 x 5 tiles at any time, which shares 11 operand panels in the die's L2 instead of
    // the 18 of two full tile rows.
    const int full = a.tiles_m / kBandRows;                 // complete bands
    const int in_full = full * kBandRows * a.tiles_n;
    int rows = kBandRows, first = 0;
    if (r >= in_full) { r -= in_full; rows = a.tiles_m - full * kBandRows; first = full * kBandRows; }
    else { const int b = r / (kBandRows * a.tiles_n); r -= b * kBandRows * a.tiles_n; first = b * kBandRows; }
    t.tj = r / rows;
    t.ti = first + (r - t.tj * rows);
  }
  return t;
}

// One tile per workgroup: workgroup L runs on die L % 8.
__device__ __forceinline__ TileId decode_tile(const GemmArgs& a) {
  const int per_xcd = gridDim.x / kXcds;
  return decode_logical(a, (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds, true);
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
// Orders the LDS traffic of one wavefront for the compiler (lanes exchange data through a region
// only this wavefront touches; the LDS unit itself executes a wavefront's accesses in order).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename T> struct Chunk;           // 16 bytes of T
template <> struct Chunk<bf16_t> { static constexpr int N = 8; typedef bf16x8 vec; };
template <> struct Chunk<float> { static constexpr int N = 4; typedef f32x4 vec; };

template <typename T, int WN, int MI, int NI>
struct Epilogue {
  static constexpr int CH = Chunk<T>::N;
  typedef typename Chunk<T>::vec vec_t;
  static constexpr int LDW = WN + 4;             // floats per staged row (+4: the two half-waves
                                                 // write rows 4 apart, keep them on different banks)
  static constexpr int CPR = WN / CH;            // chunks per row
  static constexpr int PASSES = 32 * CPR / 64;   // chunks per lane per band

  const GemmArgs& a;
  int lane, row_w0, col_w0;
  bool mirror, update, skip_w, w_vec_ok, w_pref;
  float post;
  const T* __restrict__ E;
  T* __restrict__ C;
  int wm_real, wn_real, w_is_bf16;
  void* wptr;
  vec_t ev[2][PASSES];       // E operands of the current and the next band
  bf16x8 wv[2][PASSES];      // bf16 parameters of the current and the next band (update only)

  __device__ __forceinline__ Epilogue(const GemmArgs& args, int tmat, int row0, int col0, bool mir)
      : a(args), lane(threadIdx.x & 63), row_w0(row0), col_w0(col0), mirror(mir) {
    const int mi = a.members ? a.members[tmat] : tmat;
    post = 1.0f;
    if (a.post == POST_INV) post = a.scales[mi].inv;
    else if (a.post == POST_INV2) post = a.scales[mi].inv2;
    E = a.E ? static_cast<const T*>(a.E) + (size_t)tmat * a.strideE : nullptr;
    C = static_cast<T*>(a.C) + (size_t)tmat * a.strideC;
    update = a.epilogue == EPI_UPDATE;
    wm_real = wn_real = w_is_bf16 = 0;
    skip_w = true;
    wptr = nullptr;
    if (update) {
      const MatStatic& ms = a.stat[mi];
      wm_real = ms.m; wn_real = ms.n; w_is_bf16 = ms.w_dtype;
      wptr = a.dyn[mi].w;
      skip_w = (a.scales[mi].status & 2u) != 0;
    }
    w_vec_ok = (wn_real % CH) == 0;
    // bf16 parameters whose rows are whole 16-byte chunks are fetched a band ahead
    w_pref = update && !skip_w && w_is_bf16 && CH == 8 && w_vec_ok;
  }

  // Issue the global loads band `band` needs (E chunks, and the parameter chunks of an update)
  // into slot band & 1.  Called a band ahead so the latency overlaps other work.
  template <int BAND>
  __device__ __forceinline__ void prefetch() {
    constexpr int slot = BAND & 1;
#pragma unroll
    for (int pss = 0; pss < PASSES; ++pss) {
      const int idx = pss * 64 + lane;
      const int grow = row_w0 + BAND * 32 + idx / CPR, gcol = col_w0 + (idx % CPR) * CH;
      if (E != nullptr) ev[slot][pss] = *reinterpret_cast<const vec_t*>(E + (size_t)grow * a.lde + gcol);
      if constexpr (CH == 8) {
        if (w_pref && grow < wm_real && gcol + CH <= wn_real)
          wv[slot][pss] = *reinterpret_cast<const bf16x8*>(static_cast<const bf16_t*>(wptr) +
                                                          (size_t)grow * wn_real + gcol);
      }
    }
  }

  // prefetch<0>() must have been called.  lds_f: LDS scratch of (#wavefronts x 32 x LDW) floats.
  __device__ __forceinline__ void run(f32x16 (&acc)[MI][NI], float* __restrict__ lds_f) {
    const int wave = threadIdx.x >> 6;
    float* __restrict__ stage = lds_f + wave * (32 * LDW);   // private to this wavefront
    // Every wavefront has finished reading operand tiles before any staging overwrites them.  From
    // here on a wavefront only touches its own staging rows, so no workgroup barrier (and above all
    // no fence, which would wait for the global stores in flight) is needed between bands.
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wavefront's LDS reads have returned
    __builtin_amdgcn_s_barrier();
    static_for<MI>([&](auto i) {
      constexpr int slot = i & 1;
      if constexpr (i + 1 < MI) prefetch<i + 1>();
      wave_sync();         // previous band fully consumed
      static_for<NI>([&](auto j) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
          stage[r * LDW + j * 32 + (lane & 31)] = acc[i][j][v];
        }
      });
      wave_sync();
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
          for (int e = 0; e < CH; ++e) val[e] = post * (a.alpha * val[e] + a.beta * to_f32(ev[slot][pss][e]));
        } else {
#pragma unroll
          for (int e = 0; e < CH; ++e) val[e] = post * (a.alpha * val[e]);
        }
        if (a.diag != 0.0f) {
#pragma unroll
          for (int e = 0; e < CH; ++e) val[e] += (grow == gcol + e) ? a.diag : 0.0f;
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
              wv_t w_in;
              if constexpr (CH == 8) w_in = wv[slot][pss];
              else w_in = *wp;
#pragma unroll
              for (int e = 0; e < CH; ++e) w_in[e] = (bf16_t)(a.w_keep * (float)w_in[e] - a.o_scale * to_f32(ov[e]));
              *wp = w_in;
            } else {
              f32x4* wp = reinterpret_cast<f32x4*>(static_cast<float*>(wptr) + wi);
#pragma unroll
              for (int q = 0; q < CH / 4; ++q) {
                f32x4 w4 = wp[q];
#pragma unroll
                for (int e = 0; e < 4; ++e) w4[e] = a.w_keep * w4[e] - a.o_scale * to_f32(ov[q * 4 + e]);
                wp[q] = w4;
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
        wave_sync();
        constexpr int RCH = 32 / CH;               // row-chunks per band
        constexpr int MPASSES = WN * RCH / 64;
        constexpr int RPI = 64 / RCH;              // rows of the mirrored tile one store touches: all RCH pieces
                                                   // of a row go out together (stores that touch fewer rows
                                                   // are cheaper)
#pragma unroll
        for (int pss = 0; pss < MPASSES; ++pss) {
          const int c = pss * RPI + lane % RPI, rc = lane / RPI;
          vec_t ov;
#pragma unroll
          for (int e = 0; e < CH; ++e) ov[e] = (T)stage[(rc * CH + e) * LDW + c];
          *reinterpret_cast<vec_t*>(C + (size_t)(col_w0 + c) * a.ldc + row_w0 + i * 32 + rc * CH) = ov;
        }
      }
    });
  }
};

#define MONA_AS3_EPI __attribute__((address_space(3)))
// Eight transposed LDS reads (4 rows x 16 columns of bf16 per group of 16 lanes and read): four column slabs
// of 16 (32 bytes apart) for rows r0 .. r0 + 3, and the same for rows r0 + 4 .. r0 + 7 (1024 bytes = 4 staged
// rows further on), then one wait.  A free function: an asm statement cannot name variables captured by a
// lambda.  The destination registers are written when the data returns and stay untouched until the wait,
// which is tied to them.
__device__ __forceinline__ void tr_read_8_rows(u32x2 (&lo)[4], u32x2 (&hi)[4], uint32_t addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo[0]) : "v"(addr));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:1024" : "=v"(hi[0]) : "v"(addr));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:32" : "=v"(lo[1]) : "v"(addr));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:1056" : "=v"(hi[1]) : "v"(addr));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:64" : "=v"(lo[2]) : "v"(addr));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:1088" : "=v"(hi[2]) : "v"(addr));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:96" : "=v"(lo[3]) : "v"(addr));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:1120" : "=v"(hi[3]) : "v"(addr));
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(lo[0]), "+v"(hi[0]), "+v"(lo[1]), "+v"(hi[1]), "+v"(lo[2]), "+v"(hi[2]), "+v"(lo[3]), "+v"(hi[3]));
}
// Epilogue of the persistent kernel for accumulators held TRANSPOSED (the kernel feeds the Q fragment
// as the first MFMA operand): lane l of a 32 x 32 block then holds row l % 32 of the output and, per
// group of four registers, four CONSECUTIVE columns, so a whole block row (32 rows x 64 columns of this
// wavefront) is staged with 8 ds_write_b128 instead of 32 ds_write_b32.  Four passes of 8 rows x 64
// columns follow, each lane reading 8 consecutive floats back: one 16-byte chunk of E, of C and (fused
// update) of W per lane and pass.
// Staging area per wavefront: 32 rows of 256 bytes (no padding; the 16-byte chunk index is XORed with
// row % 16, which spreads both the column-wise writes and the row-wise reads over all banks).
// Mirrored (symmetric) tiles: each pass leaves its rounded bf16 row in the 256 bytes of the fp32 row it
// has just consumed (at 32 (row % 4) bytes inside it), and ds_read_b64_tr_b16 then hands every lane 4
// consecutive rows of one column: two of them make a 16-byte piece of the transposed tile.
//
// Global loads and stores: the load counter of this target counts both, in issue order, so once a store
// is in flight a wait for a load issued after it waits for the store as well.  The E chunks
// (and the parameter chunks of the fused update) of a whole batch of NPF passes are therefore requested
// together, waited for ONCE (settle(), which also tells the compiler that these registers hold plain
// values from then on), and the stores of the passes then stream without any wait.  HAS_E is a template
// parameter for the same reason: a run-time test around the loads would make every later use look as if
// it might still be pending.
template <int MI, int NPF, int NPRE, bool UPD, bool HAS_E, bool DIAG>
struct BlockEpilogue {
  static constexpr int NI = 2, WN = 64, CH = 8, PASSES = MI * 4;
  static constexpr int kStageBytesPerWave = 32 * WN * 4;
  static_assert(NPF == 8 || NPF == 16, "settle() is written for batches of 8 or 16 passes");

  const GemmArgs& a;
  int lane, row_w0, col_w0;
  bool mirror, skip_w, w_pref;
  bool has_diag;                 // this wavefront's part of the tile holds elements of the main diagonal that get a.diag
  float c_acc, c_e;              // out = c_acc * accumulator + c_e * E  (post-scale folded in)
  // tile-relative addressing: wavefront-uniform 64-bit bases plus 32-bit lane offsets
  const char* __restrict__ Et;
  char* __restrict__ Ct;
  char* __restrict__ Cm;         // base of the mirrored tile
  uint32_t e_off, c_off;         // lane offsets (bytes) of pass 0; a wavefront tile spans < 2^32 bytes
  int wm_real, wn_real, w_is_bf16;
  void* wptr;
  u32x4 ev[HAS_E ? NPF : 1];
  u32x4 wv[UPD ? NPF : 1];     // parameter chunks, only in the launch that carries the update

  __device__ __forceinline__ BlockEpilogue(const GemmArgs& args) : a(args), lane(threadIdx.x & 63) {}

  // one wait for everything requested so far; afterwards the batch registers are ordinary values
  __device__ __forceinline__ void settle() {
    if constexpr (HAS_E) {
      asm volatile("s_waitcnt vmcnt(0)"
                   : "+v"(ev[0]), "+v"(ev[1]), "+v"(ev[2]), "+v"(ev[3]), "+v"(ev[4]), "+v"(ev[5]), "+v"(ev[6]), "+v"(ev[7]));
      if constexpr (NPF == 16)
        asm volatile("" : "+v"(ev[8]), "+v"(ev[9]), "+v"(ev[10]), "+v"(ev[11]), "+v"(ev[12]), "+v"(ev[13]),
                     "+v"(ev[14]), "+v"(ev[15]));
    }
    if constexpr (UPD) {
      static_assert(!UPD || NPF == 8, "the fused update fetches 8 passes at a time");
      asm volatile("s_waitcnt vmcnt(0)"
                   : "+v"(wv[0]), "+v"(wv[1]), "+v"(wv[2]), "+v"(wv[3]), "+v"(wv[4]), "+v"(wv[5]), "+v"(wv[6]), "+v"(wv[7]));
    }
  }

  // the same for one block row of the launch that carries the update: its block rows alternate between
  // the two halves of the batch registers, and the next row is requested only after this wait, so
  // nothing but this row's chunks (and the previous row's stores) is outstanding here
  template <int H>
  __device__ __forceinline__ void settle_half() {
    static_assert(UPD && NPF == 8, "halves of a batch of 8 passes");
    if constexpr (HAS_E)
      asm volatile("s_waitcnt vmcnt(0)"
                   : "+v"(ev[4 * H]), "+v"(ev[4 * H + 1]), "+v"(ev[4 * H + 2]), "+v"(ev[4 * H + 3]),
                     "+v"(wv[4 * H]), "+v"(wv[4 * H + 1]), "+v"(wv[4 * H + 2]), "+v"(wv[4 * H + 3]));
    else
      asm volatile("s_waitcnt vmcnt(0)" : "+v"(wv[4 * H]), "+v"(wv[4 * H + 1]), "+v"(wv[4 * H + 2]), "+v"(wv[4 * H + 3]));
  }

  __device__ __forceinline__ void begin(int tmat, int row0, int col0, bool mir) {
    row_w0 = row0; col_w0 = col0;
    mirror = UPD ? false : mir;   // the launch that carries the update is an apply: never symmetric
    // The lane number is made opaque per tile: everything the epilogue derives from it (staging and
    // global offsets) is then recomputed here, a few instructions, instead of being hoisted out of a
    // persistent kernel's tile loop and held in registers across the K loop, where there are none to spare.
    int l = threadIdx.x & 63;
    asm volatile("" : "+v"(l));
    lane = l;
    const int mi = a.members ? a.members[tmat] : tmat;
    float post = 1.0f;
    if (a.post == POST_INV) post = a.scales[mi].inv;
    else if (a.post == POST_INV2) post = a.scales[mi].inv2;
    c_acc = post * a.alpha;
    c_e = post * a.beta;
    has_diag = DIAG && a.diag != 0.0f && row0 < col0 + WN && col0 < row0 + 32 * MI;
    const int prow = lane >> 3, q = lane & 7;
    Et = HAS_E ? reinterpret_cast<const char*>(static_cast<const bf16_t*>(a.E) + (size_t)tmat * a.strideE +
                                               (size_t)row0 * a.lde + col0)
               : nullptr;
    bf16_t* const C = static_cast<bf16_t*>(a.C) + (size_t)tmat * a.strideC;
    Ct = reinterpret_cast<char*>(C + (size_t)row0 * a.ldc + col0);
    Cm = reinterpret_cast<char*>(C + (size_t)col0 * a.ldc + row0);
    e_off = 2u * (uint32_t)(prow * a.lde + q * CH);
    c_off = 2u * (uint32_t)(prow * a.ldc + q * CH);
    wm_real = wn_real = w_is_bf16 = 0;
    skip_w = true;
    wptr = nullptr;
    if constexpr (UPD) {
      const MatStatic& ms = a.stat[mi];
      wm_real = ms.m; wn_real = ms.n; w_is_bf16 = ms.w_dtype;
      wptr = a.dyn[mi].w;
      skip_w = (a.scales[mi].status & 2u) != 0;
    }
    w_pref = UPD && !skip_w && w_is_bf16 && (wn_real % CH) == 0;
  }

  // first row of pass p inside the wavefront tile: block row p / 4, rows 8 (p % 4) .. + 7
  static __device__ __forceinline__ constexpr int pass_row(int p) { return (p >> 2) * 32 + (p & 3) * 8; }

  template <int P>
  __device__ __forceinline__ void prefetch() {
    constexpr int slot = P % NPF;
    if constexpr (HAS_E) ev[slot] = *reinterpret_cast<const u32x4*>(Et + (e_off + 2u * (uint32_t)(pass_row(P) * a.lde)));
    if constexpr (UPD) {
      const int grow = row_w0 + pass_row(P) + (lane >> 3), gcol = col_w0 + (lane & 7) * CH;
      if (w_pref && grow < wm_real && gcol + CH <= wn_real)
        wv[slot] = *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(wptr) + (size_t)grow * wn_real + gcol);
    }
  }
  __device__ __forceinline__ void prefetch_first() {
    static_for<NPRE>([&](auto p) { prefetch<p>(); });
  }

  // acc[i][j]: block (i, j) of the wavefront tile, transposed operand roles (see above).
  // stage: kStageBytesPerWave bytes of LDS private to this wavefront, 256-byte aligned.
  __device__ __forceinline__ void run(f32x16 (&acc)[MI][NI], char* stage) {
    static_assert(NPRE <= NPF && PASSES % NPF == 0, "passes are fetched in batches of NPF");
    if constexpr (UPD) {
      static_for<4>([&](auto p) { prefetch<p>(); });     // block row 0; row i + 1 follows while row i is worked on
    } else {
      static_for<NPF - NPRE>([&](auto p) { prefetch<NPRE + p>(); });
    }
    if (DIAG && has_diag) {
      // (wavefront-uniform, and rare: only the poly launches of the fused schedule add a diagonal term,
      // and only in the wavefronts whose part of a diagonal tile meets the diagonal)  The term goes into
      // the accumulators, divided by their factor, so that the passes below stay as they are.
      // Register v of block (i, j) holds row 32 i + lane % 32, column 32 j + 8 (v / 4) + 4 (lane / 32) + v % 4.
      const float dv = a.diag / c_acc;
      const int d0 = row_w0 - col_w0 + (lane & 31) - 4 * (lane >> 5);
      static_for<MI>([&](auto i) {
        static_for<NI>([&](auto j) {
#pragma unroll
          for (int v = 0; v < 16; ++v)
            acc[i][j][v] += (d0 + 32 * (i - j) - 8 * (v >> 2) - (v & 3) == 0) ? dv : 0.0f;
        });
      });
    }
    const int srow = lane & 31, shalf = lane >> 5;       // staging writes: row and 4-column half
    const int prow = lane >> 3, q = lane & 7;            // passes: row inside the pass and 8-column chunk
    const uint32_t stage_addr = (uint32_t)(uintptr_t)(MONA_AS3_EPI const char*)stage;
    static_for<MI>([&](auto i) {
      wave_sync();         // previous block row fully consumed
      static_for<NI>([&](auto j) {
        static_for<4>([&](auto vg) {
          const int c = j * 8 + 2 * vg + shalf;
          f32x4 v = {acc[i][j][vg * 4 + 0], acc[i][j][vg * 4 + 1], acc[i][j][vg * 4 + 2], acc[i][j][vg * 4 + 3]};
          *reinterpret_cast<f32x4*>(stage + srow * 256 + ((c ^ (srow & 15)) << 4)) = v;
        });
      });
      wave_sync();
      // the batch this block row starts: request it (the first one was requested above) and wait once,
      // after the staging writes so that they overlap the latency
      if constexpr (UPD) {
        settle_half<i & 1>();
        if constexpr (i + 1 < MI) static_for<4>([&](auto k) { prefetch<(i + 1) * 4 + k>(); });
      } else if constexpr ((i * 4) % NPF == 0) {
        if constexpr (i > 0) static_for<NPF>([&](auto k) { prefetch<i * 4 + k>(); });
        settle();
      }
      // all reads of the block row are issued before the first result is used: one LDS round trip per
      // block row instead of one per pass (and every staged row is read before a pass overwrites part of
      // it with its bf16 row)
      f32x4 t[4][2];
      static_for<4>([&](auto pp) {
        const int r = pp * 8 + prow;
        t[pp][0] = *reinterpret_cast<const f32x4*>(stage + r * 256 + (((2 * q) ^ (r & 15)) << 4));
        t[pp][1] = *reinterpret_cast<const f32x4*>(stage + r * 256 + (((2 * q + 1) ^ (r & 15)) << 4));
      });
      // unit: the accumulator enters with factor 1 (every apply but the first), one operation less per element
      auto passes = [&](auto unit) {
      static_for<4>([&](auto pp) {
        constexpr int p = i * 4 + pp;
        constexpr int slot = p % NPF;
        const int r = pp * 8 + prow;
        const int grow = row_w0 + pass_row(p) + prow, gcol = col_w0 + q * CH;
        float val[CH];
        {
          const f32x4 t0 = t[pp][0], t1 = t[pp][1];
          val[0] = t0.x; val[1] = t0.y; val[2] = t0.z; val[3] = t0.w;
          val[4] = t1.x; val[5] = t1.y; val[6] = t1.z; val[7] = t1.w;
        }
        if constexpr (HAS_E) {
          const bf16x8 e8 = __builtin_bit_cast(bf16x8, ev[slot]);
#pragma unroll
          for (int e = 0; e < CH; ++e) {
            if constexpr (unit) val[e] = fmaf(c_e, (float)e8[e], val[e]);
            else val[e] = fmaf(c_acc, val[e], c_e * (float)e8[e]);
          }
        } else {
#pragma unroll
          for (int e = 0; e < CH; ++e) val[e] = c_acc * val[e];
        }
        bf16x8 ov;
#pragma unroll
        for (int e = 0; e < CH; ++e) ov[e] = (bf16_t)val[e];
        if (!UPD || a.store_out) *reinterpret_cast<bf16x8*>(Ct + (c_off + 2u * (uint32_t)(pass_row(p) * a.ldc))) = ov;
        // the rounded row, for the transposed store below: inside the fp32 row just read
        if (mirror) *reinterpret_cast<bf16x8*>(stage + r * 256 + (r & 3) * 32 + q * 16) = ov;
        if (UPD && !skip_w && grow < wm_real) {
          // W <- (1 - eta lambda) W - eta gamma O, O as stored in the working precision
          const size_t wi = (size_t)grow * wn_real + gcol;
          if (w_pref && gcol + CH <= wn_real) {
            bf16x8 w_in = __builtin_bit_cast(bf16x8, wv[UPD ? slot : 0]);
#pragma unroll
            for (int e = 0; e < CH; ++e) w_in[e] = (bf16_t)(a.w_keep * (float)w_in[e] - a.o_scale * (float)ov[e]);
            *reinterpret_cast<bf16x8*>(static_cast<bf16_t*>(wptr) + wi) = w_in;
          } else {
#pragma unroll
            for (int e = 0; e < CH; ++e) {
              if (gcol + e < wn_real) {
                if (w_is_bf16) {
                  bf16_t* w = static_cast<bf16_t*>(wptr) + wi + e;
                  *w = (bf16_t)(a.w_keep * (float)*w - a.o_scale * (float)ov[e]);
                } else {
                  float* w = static_cast<float*>(wptr) + wi + e;
                  *w = a.w_keep * *w - a.o_scale * (float)ov[e];
                }
              }
            }
          }
        }
      });
      };
      if (HAS_E && c_acc == 1.0f) passes(IC<1>{}); else passes(IC<0>{});
      if (mirror) {
        // 16 lanes fetch a 4 (rows) x 16 (columns) block of the bf16 rows: lane j of the group points at
        // row j / 4, columns 4 (j % 4) .. + 3 and receives the 4 rows of column j.  Group g of the wavefront
        // takes rows 8 g .. 8 g + 7 of the block row (two reads, 4 x 256 bytes apart) and, one after the
        // other, the four slabs of 16 columns: per store the four groups then write the four 16-byte pieces
        // of the same 16 rows of the mirrored tile, 64 contiguous bytes per row (measured: stores that touch
        // 16 rows cost half of stores that touch 64).
        wave_sync();
        const int j16 = lane & 15, g = lane >> 4;
        const int rr = j16 >> 2;     // (8 g + rr + 4) % 4 == rr: the staged row's offset inside its slot
        const uint32_t addr = stage_addr + (8 * g + rr) * 256 + rr * 32 + (4 * (j16 & 3)) * 2;
        u32x2 lo[4], hi[4];
        tr_read_8_rows(lo, hi, addr);
        static_for<4>([&](auto sl) {
          const u32x4 tv = {lo[sl].x, lo[sl].y, hi[sl].x, hi[sl].y};
          const int n = 16 * sl + j16;
          *reinterpret_cast<u32x4*>(Cm + 2u * ((uint32_t)(n * a.ldc) + (uint32_t)(i * 32 + g * 8))) = tv;
        });
      }
    });
  }
};

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

  Epilogue<bf16_t, WN, MI, NI> epi(a, t.mat, m0 + wm * WM, n0 + wn * WN, a.symmetric && (t.ti != t.tj));
  epi.template prefetch<0>();
  epi.run(acc, reinterpret_cast<float*>(&lds[0][0]));
}

// ---- bf16 kernel, direct-to-LDS pipeline ------------------------------------------------------
// Block tile BM x BN, WGM x WGN wavefronts of 128 x 64 each, K step 32, a ring of STAGES LDS
// stages filled straight from global memory (global_load_lds, 16 bytes per lane, no staging
// registers): 256 x 256, 8 wavefronts, 4 stages (128 KB LDS), one workgroup per CU, two wavefronts
// per SIMD.
//
// LDS layouts of one R x 32 operand tile, in 16-byte chunks:
//   row-major operand (K contiguous in memory): R rows x 4 chunks, chunk c of row r at
//     r * 4 + (c ^ ((r >> 2) & 3)); a fragment is one ds_read_b128 per lane (8 consecutive k);
//   K-major operand (stored K x R): 32 k-rows x R/8 chunks, chunk c of k-row k at
//     k * (R / 8) + (c ^ ((k & 3) << 2)); a fragment is two ds_read_b64_tr_b16 per lane: 16 lanes
//     fetch a 4 (k) x 16 (r) block and each receives the 4 k-values of one r.
// A direct load writes lane l's 16 bytes at (wave-uniform base) + 16 l, so the swizzle is applied
// by choosing which global chunk each lane fetches.
typedef short s16x4 __attribute__((ext_vector_type(4)));
#define MONA_AS1 __attribute__((address_space(1)))
#define MONA_AS3 __attribute__((address_space(3)))

// A fragment as the LDS read instructions deliver it.  The registers are written when the data
// returns, not when the read is issued, so until the matching wait they must stay exactly where
// the read instruction was told to put them: no copies, no repacking.  Each kind therefore keeps
// the destination registers of its reads as they are and is only turned into an MFMA operand
// after the wait.
struct FragR {            // row-major operand: one ds_read_b128
  u32x4 v;
  __device__ __forceinline__ bf16x8 get() const { return __builtin_bit_cast(bf16x8, v); }
};
struct FragT {            // K-major operand: two ds_read_b64_tr_b16 (k 0..3 and k 4..7 of the lane's row)
  u32x2 lo, hi;
  __device__ __forceinline__ bf16x8 get() const {
    const u32x4 v = {lo.x, lo.y, hi.x, hi.y};
    return __builtin_bit_cast(bf16x8, v);
  }
};
// s_waitcnt lgkmcnt(PENDING) tied to the fragment registers it guards, so that no consumer of those
// registers can be scheduled above the wait.
template <int PENDING>
__device__ __forceinline__ void wait_frags(FragR (&a)[4], FragR (&b)[2]) {
  asm volatile("s_waitcnt lgkmcnt(%6)"
               : "+v"(a[0].v), "+v"(a[1].v), "+v"(a[2].v), "+v"(a[3].v), "+v"(b[0].v), "+v"(b[1].v)
               : "n"(PENDING));
}
template <int PENDING>
__device__ __forceinline__ void wait_frags(FragR (&a)[4], FragT (&b)[2]) {
  asm volatile("s_waitcnt lgkmcnt(%8)"
               : "+v"(a[0].v), "+v"(a[1].v), "+v"(a[2].v), "+v"(a[3].v), "+v"(b[0].lo), "+v"(b[0].hi), "+v"(b[1].lo),
                 "+v"(b[1].hi)
               : "n"(PENDING));
}
template <int PENDING>
__device__ __forceinline__ void wait_frags(FragT (&a)[4], FragT (&b)[2]) {
  asm volatile("s_waitcnt lgkmcnt(%12)"
               : "+v"(a[0].lo), "+v"(a[0].hi), "+v"(a[1].lo), "+v"(a[1].hi), "+v"(a[2].lo), "+v"(a[2].hi), "+v"(a[3].lo),
                 "+v"(a[3].hi), "+v"(b[0].lo), "+v"(b[0].hi), "+v"(b[1].lo), "+v"(b[1].hi)
               : "n"(PENDING));
}
// reads at (address register) + (compile-time offset, below 64 KB)
template <int OFF>
__device__ __forceinline__ void lds_read(FragR& f, uint32_t addr) {
  static_assert(OFF >= 0 && OFF < 65536, "ds offset field is 16 bits");
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.v) : "v"(addr), "n"(OFF));
}
template <int OFF, int PITCH4>     // PITCH4: bytes between k-row k and k-row k + 4
__device__ __forceinline__ void lds_read_t(FragT& f, uint32_t addr) {
  static_assert(OFF >= 0 && OFF + PITCH4 < 65536, "ds offset field is 16 bits");
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.lo) : "v"(addr), "n"(OFF));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.hi) : "v"(addr), "n"(OFF + PITCH4));
}
// s_waitcnt vmcnt(n), leaving the other counters alone (gfx9 encoding)
#define MONA_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

template <int BM, int BN, int WGM, int WGN, int STAGES, int MIN_BLOCKS, bool TP, bool TQ, bool UPD, bool HAS_E, bool DIAG>
__global__ __launch_bounds__(64 * WGM * WGN, MIN_BLOCKS) void ns_gemm_bf16_dma_kernel(const GemmArgs a) {
  constexpr int BK = 32;
  constexpr int NW = WGM * WGN;
  constexpr int WM = 128, WN = 64, MI = 4, NI = 2;
  static_assert(BM == WGM * WM && BN == WGN * WN, "block tile = wavefront grid x 128 x 64");
  constexpr int P_U = BM * 4, Q_U = BN * 4;          // 16-byte units per operand tile
  constexpr int STAGE_U = P_U + Q_U;
  constexpr int NLP = P_U / (64 * NW), NLQ = Q_U / (64 * NW);   // direct loads per wavefront and stage
  constexpr int LPS = NLP + NLQ;
  static_assert(NLP * 64 * NW == P_U && NLQ * 64 * NW == Q_U, "tiles must split evenly over the wavefronts");
  constexpr int kStageFloats = NW * 32 * (WN + 4);
  static_assert(kStageFloats * 4 <= STAGES * STAGE_U * 16, "epilogue staging must fit in the operand ring");
  // the ring, and behind it what the epilogue's staging needs beyond the last stage
  constexpr int LDS_U = STAGES * STAGE_U + (NW * 8192 / 16 - STAGE_U);
  static_assert(LDS_U * 16 <= 160 * 1024, "LDS of one CU");
  __shared__ __attribute__((aligned(256))) u32x4 lds[LDS_U];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps LDS bases in SGPRs
  const int wm = wave / WGN, wn = wave % WGN;

  // ---- persistent tile walk ----
  // Workgroup b runs on die b % 8.  Every die owns one contiguous range of the matrix-major tile
  // order (tiles that share operand panels share that die's L2); its workgroups take the tiles of
  // that range round by round.
  const int total = a.tiles_per_mat * a.count;
  const int per_xcd = (total + kXcds - 1) / kXcds;
  const int xcd = blockIdx.x % kXcds, slot_in_xcd = blockIdx.x / kXcds, slots = gridDim.x / kXcds;
  auto tile_at = [&](int round) -> TileId {
    const int local = round * slots + slot_in_xcd;
    return decode_logical(a, xcd * per_xcd + local, local < per_xcd);
  };

  // ---- direct loads: per-tile lane addresses ----
  const bf16_t* gp[NLP];
  const bf16_t* gq[NLQ];
  auto set_tile = [&](const TileId& t) {
    const bf16_t* __restrict__ P = static_cast<const bf16_t*>(a.P) + (size_t)t.mat * a.strideP;
    const bf16_t* __restrict__ Q = static_cast<const bf16_t*>(a.Q) + (size_t)t.mat * a.strideQ;
    const int m0 = t.ti * BM, n0 = t.tj * BN;
    static_for<NLP>([&](auto q) {
      const int S = (wave * NLP + q) * 64 + lane;
      if constexpr (!TP) {
        const int row = S >> 2, c = (S & 3) ^ ((row >> 2) & 3);
        gp[q] = P + (size_t)(m0 + row) * a.ldp + c * 8;
      } else {
        constexpr int CPR = BM / 8;
        const int k = S / CPR, c = (S % CPR) ^ ((k & 3) << 2);
        gp[q] = P + (size_t)k * a.ldp + m0 + c * 8;
      }
    });
    static_for<NLQ>([&](auto q) {
      const int S = (wave * NLQ + q) * 64 + lane;
      if constexpr (!TQ) {
        const int row = S >> 2, c = (S & 3) ^ ((row >> 2) & 3);
        gq[q] = Q + (size_t)(n0 + row) * a.ldq + c * 8;
      } else {
        constexpr int CPR = BN / 8;
        const int k = S / CPR, c = (S % CPR) ^ ((k & 3) << 2);
        gq[q] = Q + (size_t)k * a.ldq + n0 + c * 8;
      }
    });
  };
  const size_t incp = TP ? (size_t)BK * a.ldp : (size_t)BK;   // elements per K step
  const size_t incq = TQ ? (size_t)BK * a.ldq : (size_t)BK;
  auto issue = [&](int stage, int kt) {
    u32x4* sp = lds + stage * STAGE_U;
    static_for<NLP>([&](auto q) {
      __builtin_amdgcn_global_load_lds((const MONA_AS1 void*)(gp[q] + kt * incp),
                                       (MONA_AS3 void*)(sp + (wave * NLP + q) * 64), 16, 0, 0);
    });
    static_for<NLQ>([&](auto q) {
      __builtin_amdgcn_global_load_lds((const MONA_AS1 void*)(gq[q] + kt * incq),
                                       (MONA_AS3 void*)(sp + P_U + (wave * NLQ + q) * 64), 16, 0, 0);
    });
  };

  // ---- fragment addresses, per lane ----
  // Every read is (address register) + (compile-time offset).  The offset field holds 16 bits, so
  // there is one set of address registers for stages 0-1 and one for stages 2-3 (64 KB apart); the
  // stage parity, the operand (Q tiles follow P tiles), the MFMA block and the k half go in the offset.
  const uint32_t lds_base = (uint32_t)(uintptr_t)(MONA_AS3 const char*)reinterpret_cast<const char*>(lds);
  static_assert(STAGE_U * 16 == 32768, "two stages per 64 KB");
  // row-major layout: lane's row inside a 32-row block and its swizzled chunk, one variant per k half
  const int rsw = ((lane & 31) >> 2) & 3;                 // (row >> 2) & 3, the same for every block
  uint32_t ra_addr[2][2], rb_addr[2][2];                  // [stage pair][k half]
  // K-major layout: k-row and 16-byte chunk this lane fetches for a 4 x 16 transposed block
  const int t_k = 8 * (lane >> 5) + ((lane & 15) >> 2);    // + 16 kk + 4 quad
  const int t_x = (lane & 15) >> 2;                        // k & 3 of that row: the swizzle term
  const int t_nl = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);  // r inside the 32-wide block
  uint32_t ta_addr[2][MI], tb_addr[2][NI];                // [stage pair][block]: the swizzle permutes blocks
  static_for<2>([&](auto h) {
    static_for<2>([&](auto kk) {
      const uint32_t off = (uint32_t)(((lane & 31) * 4 + ((2 * kk + (lane >> 5)) ^ rsw)) * 16);
      ra_addr[h][kk] = lds_base + h * 65536 + wm * WM * 64 + off;
      rb_addr[h][kk] = lds_base + h * 65536 + wn * WN * 64 + off;
    });
    static_for<MI>([&](auto i) {
      const int c = (wm * (WM / 8) + i * 4 + (t_nl >> 3)) ^ (t_x << 2);
      ta_addr[h][i] = lds_base + h * 65536 + (uint32_t)(t_k * (BM * 2) + c * 16 + (t_nl & 7) * 2);
    });
    static_for<NI>([&](auto j) {
      const int c = (wn * (WN / 8) + j * 4 + (t_nl >> 3)) ^ (t_x << 2);
      tb_addr[h][j] = lds_base + h * 65536 + (uint32_t)(t_k * (BN * 2) + c * 16 + (t_nl & 7) * 2);
    });
  });

  f32x16 acc[MI][NI];

  // Fragment reads are written in assembly so that their order and their count are fixed: the
  // waits below rely on LDS returning data in issue order (s_waitcnt lgkmcnt(n) = "all but the
  // last n reads have returned"), and the compiler, which cannot see that reads of one stage do not
  // touch the stages still being filled by direct loads, would otherwise wait for those loads.
  // Two register slots: while slot 0 is multiplied, slot 1 is being filled.
  typedef typename std::conditional<TP, FragT, FragR>::type FragA;
  typedef typename std::conditional<TQ, FragT, FragR>::type FragB;
  FragA fa[2][MI];
  FragB fb[2][NI];
  constexpr int kReadsA = TP ? 2 * MI : MI, kReadsB = TQ ? 2 * NI : NI;
  constexpr int kReads = kReadsA + kReadsB;          // LDS reads per slot fill
  constexpr int kPend = kReads > 15 ? 15 : kReads;   // lgkmcnt is a 4-bit counter
  auto fill = [&](auto slot, auto stage, auto kk) {
    constexpr int h = stage >> 1;
    constexpr int soff = (stage & 1) * 32768;
    static_for<MI>([&](auto i) {
      if constexpr (!TP) lds_read<soff + i * 2048>(fa[slot][i], ra_addr[h][kk]);
      else lds_read_t<soff + kk * (16 * BM * 2), 4 * BM * 2>(fa[slot][i], ta_addr[h][i]);
    });
    static_for<NI>([&](auto j) {
      if constexpr (!TQ) lds_read<soff + P_U * 16 + j * 2048>(fb[slot][j], rb_addr[h][kk]);
      else lds_read_t<soff + P_U * 16 + kk * (16 * BN * 2), 4 * BN * 2>(fb[slot][j], tb_addr[h][j]);
    });
  };
  auto arrive = [&](auto slot, auto pending) {
    static_assert(MI == 4 && NI == 2, "written for 4 x 2 blocks");
    wait_frags<pending>(fa[slot], fb[slot]);
  };
  // fresh: the first product of a tile starts from a zero accumulator operand (an inline constant)
  // instead of 128 registers cleared beforehand
  auto multiply = [&](auto slot, auto fresh) {
    static_for<MI>([&](auto i) {
      static_for<NI>([&](auto j) {
        // operand roles swapped: the block is accumulated transposed (lane = output row), which is the
        // layout the epilogue stages with 16-byte LDS writes
        if constexpr (fresh) {
          const f32x16 zero = {};
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[slot][j].get(), fa[slot][i].get(), zero, 0, 0, 0);
        } else {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[slot][j].get(), fa[slot][i].get(), acc[i][j], 0, 0, 0);
        }
      });
    });
  };

  const int KT = a.K / BK;      // a multiple of 4: K is a multiple of 128
  // One K step on stage u (compile-time).  On entry slot 0 holds (or is receiving) the first half
  // of stage u, and stages u and u + 1 are complete for every wavefront.
  //   MORE:  another stage follows: its first half is fetched while the second half is multiplied
  //   SYNC:  wait for this wavefront's loads of stage u + 2 (all but LEFT newer loads done), then meet
  //          the other wavefronts: afterwards stage u + 2 is complete and stage u is free
  //   ISSUE: request chunk kt + 4 into stage u
  auto step = [&](auto u, int kt, auto MORE, auto SYNC, auto LEFT, auto ISSUE, auto FRESH) {
    fill(IC<1>{}, u, IC<1>{});
    arrive(IC<0>{}, IC<kPend>{});
    multiply(IC<0>{}, FRESH);
    if constexpr (MORE) {
      fill(IC<0>{}, IC<(u + 1) & 3>{}, IC<0>{});
      arrive(IC<1>{}, IC<kPend>{});
    } else {
      arrive(IC<1>{}, IC<0>{});
    }
    multiply(IC<1>{}, IC<0>{});
    if constexpr (SYNC) {
      MONA_WAIT_VM(LEFT);
      __builtin_amdgcn_s_barrier();     // bare barrier: a fence here would drain every load in flight
    }
    if constexpr (ISSUE) issue(u, kt + 4);
  };

  static_assert(STAGES == 4, "the pipeline below is written for a ring of 4 stages");
  // (the launch that carries the update has no registers for an early request during the last K steps)
  typedef BlockEpilogue<MI, /*batch*/ (UPD ? 8 : 16), /*early*/ (UPD ? 0 : 2), UPD, HAS_E, DIAG> Epi;
  Epi epi(a);
  static_assert(NI == Epi::NI && (3 * STAGE_U * 16 + NW * Epi::kStageBytesPerWave) <= LDS_U * 16,
                "epilogue staging: stage 3 and the LDS behind the ring");
  // epilogue staging starts at stage 3, which the next tile's early loads (stages 0..2) leave alone
  char* const stage_f = reinterpret_cast<char*>(lds + 3 * STAGE_U) + wave * Epi::kStageBytesPerWave;

  TileId t = tile_at(0);
  if (!t.valid) return;
  set_tile(t);
  issue(0, 0);
  issue(1, 1);
  issue(2, 2);
  for (int round = 0;; ++round) {
    // entry: chunks 0..2 of tile t are in flight (or landed) in stages 0..2; stage 3 is free
    // Stores of the previous epilogue may still be in flight, and how many depends on the tile (mirrored
    // or not, with or without the update), so "all but n" cannot be counted from here on until they are
    // gone: drain everything (the loads of stages 0..2 were issued a whole epilogue ago; a variant that
    // counted the stores instead measured no faster: the time goes into the barrier below, waiting for
    // the wavefronts whose epilogue ends later).
    MONA_WAIT_VM(0);
    __builtin_amdgcn_s_barrier();
    issue(3, 3);
    fill(IC<0>{}, IC<0>{}, IC<0>{});
    int kt = 0;
    // first pass of the ring: chunk 3 is in flight alone, then the steady pattern sets in
    if (KT > 4) {
      step(IC<0>{}, 0, IC<1>{}, IC<1>{}, IC<LPS>{}, IC<1>{}, IC<1>{});   // stage 2 landed long ago; LPS = chunk 3 may fly
      step(IC<1>{}, 1, IC<1>{}, IC<1>{}, IC<LPS>{}, IC<1>{}, IC<0>{});   // chunk 3 done when only chunk 4's loads remain
      step(IC<2>{}, 2, IC<1>{}, IC<1>{}, IC<LPS>{}, IC<1>{}, IC<0>{});
      step(IC<3>{}, 3, IC<1>{}, IC<1>{}, IC<LPS>{}, IC<1>{}, IC<0>{});
      kt = 4;
      for (; kt + 4 < KT; kt += 4) {
        // in flight at each SYNC: stages u + 2 and u + 3; stage u + 2 is done when LPS loads remain
        static_for<4>([&](auto u) { step(u, kt + u, IC<1>{}, IC<1>{}, IC<LPS>{}, IC<1>{}, IC<0>{}); });
      }
    } else {
      // a tile of four steps only: no first pass to start the accumulators from zero
      static_for<MI>([&](auto i) {
        static_for<NI>([&](auto j) {
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        });
      });
    }
    // last four steps: nothing left to request
    step(IC<0>{}, kt + 0, IC<1>{}, IC<1>{}, IC<LPS>{}, IC<0>{}, IC<0>{});   // stage 2 done (its loads precede stage 3's)
    step(IC<1>{}, kt + 1, IC<1>{}, IC<1>{}, IC<0>{}, IC<0>{}, IC<0>{});     // stage 3 done
    // the first epilogue bands are requested once no wait on the load counter is left, so that
    // they arrive while the last two steps are multiplied
    // (the tile's output pointers and scales are looked up only now: nothing of the epilogue is held
    // in registers across the K loop)
    if constexpr (!UPD) {
      epi.begin(t.mat, t.ti * BM + wm * WM, t.tj * BN + wn * WN, a.symmetric && (t.tj * BN >= (t.ti + 1) * BM));
      epi.prefetch_first();
    }
    step(IC<2>{}, kt + 2, IC<1>{}, IC<0>{}, IC<0>{}, IC<0>{}, IC<0>{});
    step(IC<3>{}, kt + 3, IC<0>{}, IC<0>{}, IC<0>{}, IC<0>{}, IC<0>{});
    // every wavefront is done with the operand stages: request the next tile's first chunks into
    // stages 0..2 now, so that they travel while this tile's epilogue runs out of stage 3
    const TileId next = tile_at(round + 1);
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wavefront's fragment reads have returned
    __builtin_amdgcn_s_barrier();
    if (next.valid) {
      set_tile(next);
      issue(0, 0);
      issue(1, 1);
      issue(2, 2);
    }
    if constexpr (UPD) epi.begin(t.mat, t.ti * BM + wm * WM, t.tj * BN + wn * WN, false);
    epi.run(acc, stage_f);
    if (!next.valid) break;
    t = next;
  }
}
#undef MONA_WAIT_VM

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

  Epilogue<float, 64, 2, 2> epi(a, t.mat, m0 + wm * 64, n0 + wn * 64, a.symmetric && (t.ti != t.tj));
  epi.template prefetch<0>();
  epi.run(acc, lds_raw);
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

int device_cu_count() {
  static const int num_cus = []() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < kXcds)
      n = 256;
    return n / kXcds * kXcds;
  }();
  return num_cus;
}

hipError_t launch_ns_gemm(const GemmArgs& a, int tile, bool transP, bool transQ, bool f32, int cu_cap, hipStream_t s) {
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
  if (tile == 256 && a.tile_n == 256) {
    // persistent: one workgroup per CU walks its share of the tiles
    static const int num_cus = device_cu_count();
    // (cu_cap: the caller keeps some CUs for a kernel that runs beside this one; every workgroup of a
    // persistent launch must be resident at once or the tile walk falls into two rounds)
    const int cap = (cu_cap >= kXcds && cu_cap < num_cus) ? cu_cap / kXcds * kXcds : num_cus;
    const int pgrid = grid < cap ? grid : cap;
#define MONA_LAUNCH_DMA(TP_, TQ_, UPD_, E_)                                                                        \
  hipLaunchKernelGGL((ns_gemm_bf16_dma_kernel<256, 256, 2, 4, 4, 1, TP_, TQ_, UPD_, E_, false>), dim3(pgrid), dim3(512), 0, s, a)
    const bool upd = a.epilogue == EPI_UPDATE, has_e = a.E != nullptr;
    // the plan uses: Gram and the products of two commuting symmetric matrices (no E; both operands row-major,
    // or both K-major); poly and the apply of a wide matrix (E, both operands K-major); the apply of a tall
    // matrix (P row-major, Q K-major; with E in the literal schedule, without in the fused one); and the
    // apply that carries the update (P row-major: a K-major P leaves it no registers; with or without E)
    if (a.diag != 0.0f) {
      // only the poly launches of the fused schedule (symmetric, E, both operands K-major) add a diagonal term
      if (!(transP && transQ && !upd && has_e && a.symmetric)) return hipErrorInvalidValue;
      hipLaunchKernelGGL((ns_gemm_bf16_dma_kernel<256, 256, 2, 4, 4, 1, true, true, false, true, true>), dim3(pgrid),
                         dim3(512), 0, s, a);
    }
    else if (!transP && !transQ && !upd && !has_e) MONA_LAUNCH_DMA(false, false, false, false);
    else if (transP && transQ && !upd && !has_e) MONA_LAUNCH_DMA(true, true, false, false);
    else if (transP && transQ && !upd && has_e) MONA_LAUNCH_DMA(true, true, false, true);
    else if (!transP && transQ && !upd && has_e) MONA_LAUNCH_DMA(false, true, false, true);
    else if (!transP && transQ && !upd && !has_e) MONA_LAUNCH_DMA(false, true, false, false);
    else if (!transP && transQ && upd && has_e) MONA_LAUNCH_DMA(false, true, true, true);
    else if (!transP && transQ && upd && !has_e) MONA_LAUNCH_DMA(false, true, true, false);
    else return hipErrorInvalidValue;
#undef MONA_LAUNCH_DMA
    return hipGetLastError();
  }
  if (tile == 128) return launch_bf16<128, 128>(a, transP, transQ, grid, s);
  return hipErrorInvalidValue;
}

}  // namespace mona
