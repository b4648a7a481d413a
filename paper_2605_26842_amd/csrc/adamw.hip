// AdamW step for the parameters that are not matrices (Sec. 4.1, text above Alg. 1: embeddings,
// biases and norm gains fall back to AdamW).  The paper prints no formula; this is the published
// decoupled-weight-decay Adam:
//     m = beta1 m + (1 - beta1) g,   v = beta2 v + (1 - beta2) g^2,
//     w <- (1 - eta lambda) w - eta (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
// One fused pass over {g, m, v, w}, every array read once and written once, all tensors of the
// list in one launch (a table maps blocks to tensors).  Per element with fp32 g and fp32 w:
// reads g, m, v, w (16 B), writes m, v, w (12 B): 28 B; with bf16 w 24 B.
#include "../../include/mona.h"
#include "mona_internal.h"

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

using namespace mona;

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kChunk = 4096;      // elements per block
constexpr size_t kAlign = 256;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  const int rc = api_fail(code, fmt, ap);
  va_end(ap);
  return rc;
}
#define HIP_TRY(expr)                                                                       \
  do {                                                                                      \
    hipError_t e__ = (expr);                                                                \
    if (e__ != hipSuccess) return fail(MONA_EHIP, "%s: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

struct VecStatic {
  float* m;          // first moment, fp32
  float* v;          // second moment, fp32
  int64_t n;         // elements
  int32_t w_dtype, g_dtype;
};
struct VecDynamic {
  void* w;
  const void* g;
};
struct VecBlock {
  int32_t vec;       // tensor index
  int32_t chunk;     // chunk index inside that tensor
};
struct AdamCoef {
  float beta1, one_minus_beta1, beta2, one_minus_beta2;
  float inv_bias1, inv_bias2;   // 1 / (1 - beta1^t), 1 / (1 - beta2^t)
  float eps, lr, keep;          // keep = 1 - eta lambda
};

__device__ __forceinline__ f32x4 ld4(const float* p) { return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p)); }
__device__ __forceinline__ f32x4 ld4(const bf16_t* p) {
  const bf16x4 v = __builtin_nontemporal_load(reinterpret_cast<const bf16x4*>(p));
  return f32x4{(float)v.x, (float)v.y, (float)v.z, (float)v.w};
}
__device__ __forceinline__ void st4(float* p, f32x4 v) { __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p)); }
__device__ __forceinline__ void st4(bf16_t* p, f32x4 v) {
  const bf16x4 r = {(bf16_t)v.x, (bf16_t)v.y, (bf16_t)v.z, (bf16_t)v.w};   // round to nearest even
  __builtin_nontemporal_store(r, reinterpret_cast<bf16x4*>(p));
}

__device__ __forceinline__ float adamw_element(float g, float& m, float& v, float w, const AdamCoef& c) {
  m = c.beta1 * m + c.one_minus_beta1 * g;
  v = c.beta2 * v + c.one_minus_beta2 * g * g;
  const float mhat = m * c.inv_bias1;
  const float vhat = v * c.inv_bias2;
  return c.keep * w - c.lr * (mhat / (sqrtf(vhat) + c.eps));
}

template <typename GT, typename WT>
__global__ __launch_bounds__(kThreads) void adamw_kernel(const VecStatic* __restrict__ stat,
                                                         const VecDynamic* __restrict__ dyn,
                                                         const VecBlock* __restrict__ work, AdamCoef c,
                                                         int want_g, int want_w) {
  const VecBlock bw = work[blockIdx.x];
  const VecStatic vs = stat[bw.vec];
  if (vs.g_dtype != want_g || vs.w_dtype != want_w) return;   // another instantiation's tensor
  const GT* __restrict__ g = static_cast<const GT*>(dyn[bw.vec].g);
  WT* __restrict__ w = static_cast<WT*>(dyn[bw.vec].w);
  float* __restrict__ mo = vs.m;
  float* __restrict__ vo = vs.v;
  const int64_t base = (int64_t)bw.chunk * kChunk;
  const int count = (int)min((int64_t)kChunk, vs.n - base);
  const int quads = count >> 2;     // a chunk starts 16-byte aligned in every array
  constexpr int kIter = kChunk / (kThreads * 4);
  f32x4 vg[kIter], vm[kIter], vv[kIter], vw[kIter];
#pragma unroll
  for (int it = 0; it < kIter; ++it) {
    const int q = it * kThreads + threadIdx.x;
    if (q < quads) {
      const int64_t i = base + (int64_t)q * 4;
      vg[it] = ld4(g + i); vm[it] = ld4(mo + i); vv[it] = ld4(vo + i); vw[it] = ld4(w + i);
    }
  }
#pragma unroll
  for (int it = 0; it < kIter; ++it) {
    const int q = it * kThreads + threadIdx.x;
    if (q < quads) {
      const int64_t i = base + (int64_t)q * 4;
      float m4[4] = {vm[it].x, vm[it].y, vm[it].z, vm[it].w};
      float v4[4] = {vv[it].x, vv[it].y, vv[it].z, vv[it].w};
      const float g4[4] = {vg[it].x, vg[it].y, vg[it].z, vg[it].w};
      const float w4[4] = {vw[it].x, vw[it].y, vw[it].z, vw[it].w};
      float n4[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) n4[e] = adamw_element(g4[e], m4[e], v4[e], w4[e], c);
      st4(mo + i, f32x4{m4[0], m4[1], m4[2], m4[3]});
      st4(vo + i, f32x4{v4[0], v4[1], v4[2], v4[3]});
      st4(w + i, f32x4{n4[0], n4[1], n4[2], n4[3]});
    }
  }
  // ragged tail of the tensor's last chunk
  const int t = quads * 4 + threadIdx.x;
  if (threadIdx.x < 4 && t < count) {
    const int64_t i = base + t;
    float m = mo[i], v = vo[i];
    const float wn = adamw_element((float)g[i], m, v, (float)w[i], c);
    mo[i] = m; vo[i] = v; w[i] = (WT)wn;
  }
}

struct Layout {
  int count = 0;
  std::vector<size_t> m_off, v_off;
  size_t state_bytes = 0;
  size_t stat_off = 0, dyn_off = 0, blocks_off = 0, total = 0;
  std::vector<VecBlock> blocks;
  bool has[2][2] = {{false, false}, {false, false}};   // [g dtype][w dtype] present in the list
};

int check_vecs(const mona_vector* vecs, int32_t count, bool need_ptrs) {
  if (!vecs) return fail(MONA_EINVAL, "vecs is NULL");
  if (count < 1) return fail(MONA_EINVAL, "count must be >= 1 (got %d)", count);
  for (int i = 0; i < count; ++i) {
    const mona_vector& q = vecs[i];
    if (q.n < 1) return fail(MONA_EINVAL, "tensor %d: n must be >= 1 (got %lld)", i, (long long)q.n);
    if (q.n > ((int64_t)1 << 40)) return fail(MONA_EINVAL, "tensor %d: n must be at most 2^40", i);
    if ((q.w_dtype != MONA_F32 && q.w_dtype != MONA_BF16) || (q.g_dtype != MONA_F32 && q.g_dtype != MONA_BF16))
      return fail(MONA_EINVAL, "tensor %d: dtype must be MONA_F32 or MONA_BF16", i);
    if (need_ptrs) {
      if (!q.w || !q.g) return fail(MONA_EINVAL, "tensor %d: w and g must not be NULL", i);
      if (((uintptr_t)q.w & 15) || ((uintptr_t)q.g & 15))
        return fail(MONA_EINVAL, "tensor %d: w and g must be 16-byte aligned", i);
    }
  }
  return MONA_OK;
}

int build_layout(const mona_vector* vecs, int count, Layout& L) {
  L.count = count;
  size_t off = 0;
  L.m_off.resize(count);
  L.v_off.resize(count);
  for (int i = 0; i < count; ++i) {
    L.m_off[i] = off; off = align_up(off + (size_t)vecs[i].n * 4);
    L.v_off[i] = off; off = align_up(off + (size_t)vecs[i].n * 4);
  }
  L.state_bytes = off;
  int64_t nblocks = 0;
  for (int i = 0; i < count; ++i) nblocks += (vecs[i].n + kChunk - 1) / kChunk;
  if (nblocks > 0x7fffff00LL) return fail(MONA_EINVAL, "too many elements for one launch");
  L.blocks.reserve((size_t)nblocks);
  for (int i = 0; i < count; ++i) {
    const int nb = (int)((vecs[i].n + kChunk - 1) / kChunk);
    for (int c = 0; c < nb; ++c) L.blocks.push_back(VecBlock{i, c});
    L.has[vecs[i].g_dtype][vecs[i].w_dtype] = true;
  }
  L.stat_off = off;   off = align_up(off + sizeof(VecStatic) * count);
  L.dyn_off = off;    off = align_up(off + sizeof(VecDynamic) * count);
  L.blocks_off = off; off = align_up(off + sizeof(VecBlock) * L.blocks.size());
  L.total = off;
  return MONA_OK;
}

constexpr int kRing = 4;

}  // namespace

struct mona_adamw_state {
  Layout L;
  std::vector<mona_vector> vecs;
  char* arena = nullptr;
  int64_t t = 0;
  VecDynamic* ring[kRing] = {nullptr, nullptr, nullptr, nullptr};
  hipEvent_t ring_ev[kRing];
  bool ring_used[kRing] = {false, false, false, false};
  int ring_next = 0;
  std::vector<VecDynamic> last_dyn;
  bool dyn_valid = false;
};

namespace {
void destroy(mona_adamw_state* st) {
  for (int i = 0; i < kRing; ++i) {
    if (st->ring_used[i]) (void)hipEventSynchronize(st->ring_ev[i]);
    if (st->ring[i]) { (void)hipHostFree(st->ring[i]); (void)hipEventDestroy(st->ring_ev[i]); }
  }
  delete st;
}
}  // namespace

extern "C" {

int mona_adamw_state_size(const mona_vector* vecs, int32_t count, size_t* bytes_out) {
  if (!bytes_out) return fail(MONA_EINVAL, "bytes_out is NULL");
  int rc = check_vecs(vecs, count, false);
  if (rc) return rc;
  Layout L;
  rc = build_layout(vecs, count, L);
  if (rc) return rc;
  *bytes_out = L.total;
  return MONA_OK;
}

int mona_adamw_init_state(const mona_vector* vecs, int32_t count, void* arena, size_t arena_bytes, void* stream,
                          mona_adamw_state** out) {
  if (!out) return fail(MONA_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = check_vecs(vecs, count, false);
  if (rc) return rc;
  if (!arena) return fail(MONA_EINVAL, "arena is NULL");
  if ((uintptr_t)arena % kAlign) return fail(MONA_EINVAL, "arena must be 256-byte aligned");
  mona_adamw_state* st = new (std::nothrow) mona_adamw_state();
  if (!st) return fail(MONA_ENOMEM, "host allocation failed");
  rc = build_layout(vecs, count, st->L);
  if (rc) { delete st; return rc; }
  const Layout& L = st->L;
  if (arena_bytes < L.total) {
    const size_t need = L.total;
    delete st;
    return fail(MONA_ENOMEM, "arena too small: %zu bytes given, %zu needed", arena_bytes, need);
  }
  st->vecs.assign(vecs, vecs + count);
  st->arena = static_cast<char*>(arena);
  hipStream_t s = static_cast<hipStream_t>(stream);
#define INIT_TRY(expr)                                                                  \
  do {                                                                                  \
    hipError_t e__ = (expr);                                                            \
    if (e__ != hipSuccess) {                                                            \
      destroy(st);                                                                      \
      return fail(MONA_EHIP, "%s: %s", #expr, hipGetErrorString(e__));                  \
    }                                                                                   \
  } while (0)
  for (int i = 0; i < kRing; ++i) {
    void* p = nullptr;
    INIT_TRY(hipHostMalloc(&p, sizeof(VecDynamic) * (size_t)count, hipHostMallocDefault));
    hipError_t e = hipEventCreateWithFlags(&st->ring_ev[i], hipEventDisableTiming);
    if (e != hipSuccess) {
      (void)hipHostFree(p);
      destroy(st);
      return fail(MONA_EHIP, "hipEventCreate: %s", hipGetErrorString(e));
    }
    st->ring[i] = static_cast<VecDynamic*>(p);
  }
  INIT_TRY(launch_fill_zero(st->arena, L.state_bytes, s));   // m_0 = v_0 = 0
  std::vector<VecStatic> stat(count);
  for (int i = 0; i < count; ++i) {
    stat[i].m = reinterpret_cast<float*>(st->arena + L.m_off[i]);
    stat[i].v = reinterpret_cast<float*>(st->arena + L.v_off[i]);
    stat[i].n = vecs[i].n;
    stat[i].w_dtype = vecs[i].w_dtype;
    stat[i].g_dtype = vecs[i].g_dtype;
  }
  INIT_TRY(hipMemcpyAsync(st->arena + L.stat_off, stat.data(), sizeof(VecStatic) * count, hipMemcpyHostToDevice, s));
  INIT_TRY(hipMemcpyAsync(st->arena + L.blocks_off, L.blocks.data(), sizeof(VecBlock) * L.blocks.size(),
                          hipMemcpyHostToDevice, s));
  INIT_TRY(hipStreamSynchronize(s));   // the host vectors above leave scope
#undef INIT_TRY
  *out = st;
  return MONA_OK;
}

int mona_adamw_step(mona_adamw_state* st, const mona_vector* vecs, int32_t count, const mona_adamw_hparams* hp,
                    void* stream) {
  if (!st) return fail(MONA_EINVAL, "state is NULL");
  int rc = check_vecs(vecs, count, true);
  if (rc) return rc;
  if (!hp) return fail(MONA_EINVAL, "hparams is NULL");
  if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) || !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f))
    return fail(MONA_EINVAL, "beta1 and beta2 must lie in [0, 1)");
  if (!std::isfinite(hp->lr) || !std::isfinite(hp->weight_decay) || !std::isfinite(hp->eps) || hp->eps < 0.0f)
    return fail(MONA_EINVAL, "hyper-parameters must be finite (and eps >= 0)");
  const Layout& L = st->L;
  if (count != L.count) return fail(MONA_ESHAPE, "count %d differs from %d at init", count, L.count);
  for (int i = 0; i < count; ++i) {
    const mona_vector& a = vecs[i];
    const mona_vector& b = st->vecs[i];
    if (a.n != b.n || a.w_dtype != b.w_dtype || a.g_dtype != b.g_dtype)
      return fail(MONA_ESHAPE, "tensor %d: size or dtype differs from init", i);
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  bool changed = !st->dyn_valid;
  if (!changed)
    for (int i = 0; i < count; ++i)
      if (st->last_dyn[i].w != vecs[i].w || st->last_dyn[i].g != vecs[i].g) { changed = true; break; }
  if (changed) {
    const int slot = st->ring_next;
    if (st->ring_used[slot]) HIP_TRY(hipEventSynchronize(st->ring_ev[slot]));
    st->last_dyn.resize(count);
    for (int i = 0; i < count; ++i) {
      st->last_dyn[i].w = vecs[i].w;
      st->last_dyn[i].g = vecs[i].g;
      st->ring[slot][i] = st->last_dyn[i];
    }
    HIP_TRY(hipMemcpyAsync(st->arena + L.dyn_off, st->ring[slot], sizeof(VecDynamic) * count, hipMemcpyHostToDevice, s));
    HIP_TRY(hipEventRecord(st->ring_ev[slot], s));
    st->ring_used[slot] = true;
    st->ring_next = (slot + 1) % kRing;
    st->dyn_valid = true;
  }
  const int64_t t = st->t + 1;
  AdamCoef c;
  c.beta1 = hp->beta1; c.one_minus_beta1 = 1.0f - hp->beta1;
  c.beta2 = hp->beta2; c.one_minus_beta2 = 1.0f - hp->beta2;
  // bias corrections in double on the host: beta^t for large t is not a job for fp32
  c.inv_bias1 = (float)(1.0 / (1.0 - std::pow((double)hp->beta1, (double)t)));
  c.inv_bias2 = (float)(1.0 / (1.0 - std::pow((double)hp->beta2, (double)t)));
  c.eps = hp->eps; c.lr = hp->lr; c.keep = 1.0f - hp->lr * hp->weight_decay;
  const VecStatic* stat = reinterpret_cast<const VecStatic*>(st->arena + L.stat_off);
  const VecDynamic* dyn = reinterpret_cast<const VecDynamic*>(st->arena + L.dyn_off);
  const VecBlock* blocks = reinterpret_cast<const VecBlock*>(st->arena + L.blocks_off);
  const int nb = (int)L.blocks.size();
  // one launch per (gradient dtype, parameter dtype) pair present; blocks of other tensors return at once
  if (L.has[MONA_F32][MONA_F32])
    hipLaunchKernelGGL((adamw_kernel<float, float>), dim3(nb), dim3(kThreads), 0, s, stat, dyn, blocks, c, MONA_F32, MONA_F32);
  if (L.has[MONA_F32][MONA_BF16])
    hipLaunchKernelGGL((adamw_kernel<float, bf16_t>), dim3(nb), dim3(kThreads), 0, s, stat, dyn, blocks, c, MONA_F32, MONA_BF16);
  if (L.has[MONA_BF16][MONA_F32])
    hipLaunchKernelGGL((adamw_kernel<bf16_t, float>), dim3(nb), dim3(kThreads), 0, s, stat, dyn, blocks, c, MONA_BF16, MONA_F32);
  if (L.has[MONA_BF16][MONA_BF16])
    hipLaunchKernelGGL((adamw_kernel<bf16_t, bf16_t>), dim3(nb), dim3(kThreads), 0, s, stat, dyn, blocks, c, MONA_BF16, MONA_BF16);
  HIP_TRY(hipGetLastError());
  st->t = t;
  return MONA_OK;
}

int mona_adamw_free_state(mona_adamw_state* st) {
  if (st) destroy(st);
  return MONA_OK;
}

int mona_adamw_state_view(mona_adamw_state* st, int32_t i, int32_t kind, void** dev_ptr, int64_t* n_out) {
  if (!st || !dev_ptr || !n_out) return fail(MONA_EINVAL, "state, dev_ptr or n_out is NULL");
  if (i < 0 || i >= st->L.count) return fail(MONA_EINVAL, "tensor index %d out of range [0, %d)", i, st->L.count);
  if (kind == MONA_ADAMW_VIEW_M) *dev_ptr = st->arena + st->L.m_off[i];
  else if (kind == MONA_ADAMW_VIEW_V) *dev_ptr = st->arena + st->L.v_off[i];
  else return fail(MONA_EINVAL, "unknown view kind %d", kind);
  *n_out = st->vecs[i].n;
  return MONA_OK;
}

int mona_adamw_state_export_size(mona_adamw_state* st, size_t* bytes_out) {
  if (!st || !bytes_out) return fail(MONA_EINVAL, "state or bytes_out is NULL");
  *bytes_out = st->L.state_bytes;
  return MONA_OK;
}

int mona_adamw_state_export(mona_adamw_state* st, void* dst, size_t dst_bytes, void* stream) {
  if (!st || !dst) return fail(MONA_EINVAL, "state or dst is NULL");
  if (dst_bytes < st->L.state_bytes) return fail(MONA_ENOMEM, "dst too small: %zu < %zu", dst_bytes, st->L.state_bytes);
  HIP_TRY(hipMemcpyAsync(dst, st->arena, st->L.state_bytes, hipMemcpyDeviceToDevice, static_cast<hipStream_t>(stream)));
  return MONA_OK;
}

int mona_adamw_state_import(mona_adamw_state* st, const void* src, size_t src_bytes, int64_t step_count, void* stream) {
  if (!st || !src) return fail(MONA_EINVAL, "state or src is NULL");
  if (src_bytes != st->L.state_bytes)
    return fail(MONA_ESHAPE, "checkpoint holds %zu bytes, this state needs %zu", src_bytes, st->L.state_bytes);
  if (step_count < 0) return fail(MONA_EINVAL, "step_count must be >= 0");
  HIP_TRY(hipMemcpyAsync(st->arena, src, st->L.state_bytes, hipMemcpyDeviceToDevice, static_cast<hipStream_t>(stream)));
  st->t = step_count;
  return MONA_OK;
}

int mona_adamw_state_step_count(mona_adamw_state* st, int64_t* t_out) {
  if (!st || !t_out) return fail(MONA_EINVAL, "state or t_out is NULL");
  *t_out = st->t;
  return MONA_OK;
}

}  // extern "C"
