// Host side of libmona: argument checking, arena layout, shape grouping and the launch plan
// of one MONA step (Alg. 1).  All arithmetic happens in the kernels of state_update.hip and
// ns_gemm.hip; this file only decides what is launched on which buffers.
#include "../../include/mona.h"
#include "mona_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace mona;

namespace {
thread_local std::string g_err;
}

namespace mona {
int api_fail(int code, const char* fmt, va_list ap) {
  char buf[512];
  vsnprintf(buf, sizeof buf, fmt, ap);
  g_err = buf;
  return code;
}
}  // namespace mona

namespace {

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

constexpr size_t kAlign = 256;
constexpr int kSmallSideF32 = 64;
constexpr double kFusedMaxStart = 0.0438;  // largest 1 / sqrt(p) + 1 / sqrt(q) for which the automatic choice fuses three iterations
constexpr int kPairsMinShortSide = 1024;   // padded short side from which it fuses pairs of iterations otherwise
size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }
int round_up(int v, int a) { return (v + a - 1) / a * a; }

enum OpKind { OP_GRAM = 0, OP_POLY = 1, OP_APPLY = 2, OP_SYMPROD = 3 };

struct Group {
  int m = 0, n = 0;          // native shape
  bool tall = false;         // m > n: Gram matrix on the column side
  int rows_pad = 0, cols_pad = 0;  // padded native shape of the working copies
  int p_pad = 0;             // padded short side
  int gran = 128;            // padding granularity (largest tile usable)
  bool f32 = false;          // products of this group run in fp32 (else bf16 operands)
  bool large_with_company = false;  // 256 x 256 tiles even for launches of few tiles (set when the state is built)
  int esize = 2;             // bytes per element of this group's working copies
  std::vector<int> members;  // matrix indices
  int fused = 0;             // Newton-Schulz iterations taken in chunks on the p x p side (see OpBuilder):
                             // 0 literal, 1 chunks of two, 2 a chunk of three and then chunks of two
  int npp = 2;               // p x p working matrices: S and B (literal schedule) or S, S', U, Q, R, R' (fused)
  int o_buf = 1;             // which ping-pong buffer holds O_k of the last step
  size_t x_off[2] = {0, 0};  // byte offsets in the arena: ping-pong X buffers
  size_t pp_off[6] = {0, 0, 0, 0, 0, 0};
  size_t members_off = 0;
  int64_t x_stride = 0, s_stride = 0;  // elements per matrix
};

struct Layout {
  int count = 0;
  int ssize = 4;             // bytes per element of the stored G_{k-1}, A (or C)
  bool one_buffer = false;   // no G_{k-1}; acc_off holds C
  bool caller_slot = false;  // G_{k-1} is kept by the caller (streaming variant)
  bool external_state = false;  // G_{k-1}, A and M live in arrays of the caller's, not in the arena
  std::vector<size_t> gprev_off, acc_off, mom_off;
  size_t state_begin = 0, state_bytes = 0;     // persistent {G_prev, A, M}
  size_t work_begin = 0, work_bytes = 0;       // X, S, B of every group (zeroed once)
  size_t stat_off = 0, dyn_off = 0, scales_off = 0, partials_off = 0, blocks_off = 0, optr_off = 0;
  size_t total = 0;
  std::vector<Group> groups;
  std::vector<int> group_of, rank_in_group;
  std::vector<BlockWork> blocks;       // ordered: fp32-gradient matrices first, then bf16
  std::vector<int> first_block, num_blocks;
  // The block table is ordered: early groups (fp32-gradient matrices, then bf16), then the late group (same).
  int range_end[4] = {0, 0, 0, 0};     // ends of those four ranges of blocks
  std::vector<int> lane_of_group;      // group index -> lane (stream) its products run on
  int lanes = 1;
  int late_group = -1;                 // group whose elementwise pass runs beside the products of the others
  std::vector<int32_t> order;          // matrix indices: early matrices, then those of the late group
  int num_early = 0;
  size_t order_off = 0;
};

int check_mats(const mona_matrix* mats, int32_t count, bool need_ptrs) {
  if (!mats) return fail(MONA_EINVAL, "mats is NULL");
  if (count < 1) return fail(MONA_EINVAL, "count must be >= 1 (got %d)", count);
  for (int i = 0; i < count; ++i) {
    const mona_matrix& q = mats[i];
    if (q.m < 1 || q.n < 1) return fail(MONA_EINVAL, "matrix %d: m and n must be >= 1 (got %d x %d)", i, q.m, q.n);
    if (q.m > (1 << 30) || q.n > (1 << 30))   // sides are rounded up to tile multiples in 32-bit arithmetic
      return fail(MONA_EINVAL, "matrix %d: m and n must each be at most 2^30 (got %d x %d)", i, q.m, q.n);
    if ((int64_t)q.m * q.n >= (int64_t)1 << 31)
      return fail(MONA_EINVAL, "matrix %d: m * n must be below 2^31 (got %d x %d)", i, q.m, q.n);
    if ((q.w_dtype != MONA_F32 && q.w_dtype != MONA_BF16) || (q.g_dtype != MONA_F32 && q.g_dtype != MONA_BF16))
      return fail(MONA_EINVAL, "matrix %d: dtype must be MONA_F32 or MONA_BF16", i);
    if (need_ptrs) {
      if (!q.w || !q.g) return fail(MONA_EINVAL, "matrix %d: w and g must not be NULL", i);
      if (((uintptr_t)q.w & 15) || ((uintptr_t)q.g & 15))
        return fail(MONA_EINVAL, "matrix %d: w and g must be 16-byte aligned", i);
    }
  }
  return MONA_OK;
}

int check_opts(const mona_options* o, mona_options* out) {
  mona_options z;
  memset(&z, 0, sizeof z);
  if (o) z = *o;
  if (z.ns_precision != 0 && z.ns_precision != 1) return fail(MONA_EINVAL, "ns_precision must be 0 or 1");
  if (z.state_dtype != MONA_F32 && z.state_dtype != MONA_BF16)
    return fail(MONA_EINVAL, "state_dtype must be MONA_F32 or MONA_BF16");
  if (z.accel_form != MONA_ACCEL_TWO_BUFFER && z.accel_form != MONA_ACCEL_ONE_BUFFER &&
      z.accel_form != MONA_ACCEL_CALLER_SLOT)
    return fail(MONA_EINVAL, "accel_form must be MONA_ACCEL_TWO_BUFFER, MONA_ACCEL_ONE_BUFFER or MONA_ACCEL_CALLER_SLOT");
  if (z.max_streams < 0 || z.max_streams > 8) return fail(MONA_EINVAL, "max_streams must lie in [0, 8]");
  if (z.ns_schedule != MONA_NS_SCHEDULE_AUTO && z.ns_schedule != MONA_NS_SCHEDULE_LITERAL &&
      z.ns_schedule != MONA_NS_SCHEDULE_FUSED && z.ns_schedule != MONA_NS_SCHEDULE_PAIRS)
    return fail(MONA_EINVAL, "ns_schedule must be MONA_NS_SCHEDULE_AUTO, _LITERAL, _FUSED or _PAIRS");
  if (z.overlap != MONA_OVERLAP_OFF && z.overlap != MONA_OVERLAP_LATE_GROUP)
    return fail(MONA_EINVAL, "overlap must be MONA_OVERLAP_OFF or MONA_OVERLAP_LATE_GROUP");
  for (int r : z.reserved)
    if (r != 0) return fail(MONA_EINVAL, "reserved option fields must be 0");
  *out = z;
  return MONA_OK;
}

constexpr int kRing = 4;
constexpr int kProfSets = 32;
constexpr int kDefaultLanes = 4;   // streams the shape groups of one step are spread over
// launches of at least this many tiles keep 256 CUs busy for six rounds or more.  Measured: with the limit at
// 512 or 768 mid-sized groups (a bank of 64 experts of 1024 x 2048) lose 4 % by waiting for each other; at
// 3072 the two expert groups of a 128-expert layer run side by side and lose 5 % to each other's L2 traffic.
constexpr long long kBigLaunchTiles = 1536;
constexpr long long kChipTiles = 256;      // one tile per CU
// CUs the late group's elementwise pass keeps to itself (a quarter of the chip): the HBM-bound pass still
// moves 2.8 TB/s there, and the power-limited products lose 13 % on the other three quarters (measured).
constexpr int kOverlapCuShare = 4;
constexpr double kSlowPassBytesPerSec = 2.8e12, kProductFlopPerSec = 1.0e15, kProductSlowdown = 1.13;

struct TileShape { int bm, bn; };

// block tile used by one product of a group
TileShape pick_tile(const Group& g, int kind, int count) {
  if (g.f32 || g.gran < 256) return {128, 128};
  long long tiles;
  if (kind == OP_APPLY) {
    tiles = (long long)(g.rows_pad / 256) * (g.cols_pad / 256) * count;
  } else {
    const long long t = g.p_pad / 256;
    tiles = t * (t + 1) / 2 * count;
  }
  // too few large tiles to fill 256 CUs, unless groups running beside this one make up for it
  if (tiles < 192 && !g.large_with_company) return {128, 128};
  return {256, 256};
}

// tiles one product launch of a group computes
long long launch_tiles(const Group& g, int kind, TileShape tile, int count) {
  if (kind == OP_APPLY) return (long long)(g.rows_pad / tile.bm) * (g.cols_pad / tile.bn) * count;
  const long long t = g.p_pad / tile.bm;
  return t * (t + 1) / 2 * count;
}


// Streams and order of the step.
//
// Lanes.  A group whose every launch covers the chip many times over gains nothing from company (two
// persistent kernels sharing the CUs only disturb each other's L2 reuse: measured slower), so such groups
// stay in a row on the caller's stream; the others, sorted by work, each go to the least loaded lane.
//
// Late group (on request: mona_options.overlap).  The elementwise pass is bound by HBM and leaves the matrix
// units idle; the products are bound by the matrix units (and by power) and leave HBM half idle.  When the
// groups in the row are several, the elementwise pass of the one with the most elements is taken out of the
// common pass and runs on a stream of its own, confined to a quarter of the CUs, beside the products of the
// other groups, which keep to the remaining three quarters; its own products come last.  Taken only where
// the products of the other groups last about as long as that slowed-down pass, so that it is hidden
// completely.  Measured (388-matrix layer): the pass is hidden, but the products beside it run 10 % slower
// (13 % from the CUs they give up, the rest from sharing HBM), which leaves 3.6 % of the step; not the default.
void plan_lanes(Layout& L, const mona_options& opt) {
  const int want = opt.max_streams == 0 ? kDefaultLanes : opt.max_streams;
  L.lanes = std::max(1, std::min<int>(want, (int)L.groups.size()));
  std::vector<std::pair<double, int>> order;
  std::vector<double> load(L.lanes, 0.0);
  L.lane_of_group.assign(L.groups.size(), 0);
  L.late_group = -1;
  std::vector<long long> fewest_of(L.groups.size(), 0);
  std::vector<int> row;
  bool any_big = false;
  for (size_t gi = 0; gi < L.groups.size(); ++gi) {
    const Group& g = L.groups[gi];
    long long fewest = -1;
    for (int kind = OP_GRAM; kind <= OP_APPLY; ++kind) {
      const long long t = launch_tiles(g, kind, pick_tile(g, kind, (int)g.members.size()), (int)g.members.size());
      if (fewest < 0 || t < fewest) fewest = t;
    }
    fewest_of[gi] = fewest;
    any_big = any_big || fewest >= kBigLaunchTiles;
  }
  std::vector<double> work_of(L.groups.size(), 0.0);
  for (size_t gi = 0; gi < L.groups.size(); ++gi) {
    const Group& g = L.groups[gi];
    const double p = std::min(g.rows_pad, g.cols_pad), q = std::max(g.rows_pad, g.cols_pad);
    // flop of five iterations on the symmetric count: literal 5 (3 p^2 q + p^3), chunks (3, 2), chunks (2, 2, 1)
    const double per = g.fused == 2 ? 6.0 * p * p * q + 14.0 * p * p * p
                       : g.fused == 1 ? 9.0 * p * p * q + 11.0 * p * p * p : 5.0 * (3.0 * p * p * q + p * p * p);
    const double work = per * (double)g.members.size();
    work_of[gi] = work;
    // Beside a group that keeps the caller's stream, only groups too small to fill the chip by
    // themselves go to the side streams (their launch latency hides behind the large group); a
    // mid-sized group there gained 0.3 % at most (4 squares of 4096 beside 384 experts), and in a row
    // the per-launch times of a profile add up to the phase time.
    const bool in_row = fewest_of[gi] >= kBigLaunchTiles || (any_big && fewest_of[gi] >= kChipTiles);
    if (in_row) { load[0] += work; row.push_back((int)gi); }
    else order.emplace_back(-work, (int)gi);
  }
  std::sort(order.begin(), order.end());
  for (auto& pr : order) {
    const int lane = (int)(std::min_element(load.begin(), load.end()) - load.begin());
    L.lane_of_group[pr.second] = lane;
    load[lane] += -pr.first;
  }
  // The groups on the lanes run side by side.  When their launches, taken together, put a large tile
  // on at least half of the CUs, each of them uses the large-tile kernel even where its own launch
  // alone would be too small for it (measured on one dense block of hidden size 2048: 2.43 against
  // 2.80 ms per step).
  if (L.lanes > 1) {
    long long together = 0;
    for (auto& pr : order) {
      Group& g = L.groups[pr.second];
      if (g.f32 || g.gran < 256) continue;
      long long fewest = -1;
      for (int kind = OP_GRAM; kind <= OP_APPLY; ++kind) {
        const long long t = launch_tiles(g, kind, TileShape{256, 256}, (int)g.members.size());
        if (fewest < 0 || t < fewest) fewest = t;
      }
      together += fewest;
    }
    if (together >= 128)
      for (auto& pr : order) L.groups[pr.second].large_with_company = true;
  }
  if (opt.overlap == MONA_OVERLAP_LATE_GROUP && row.size() >= 2 && !L.external_state) {
    int late = -1;
    double most = 0.0, others = 0.0;
    auto elems = [&](int gi) { return (double)L.groups[gi].m * L.groups[gi].n * (double)L.groups[gi].members.size(); };
    for (int gi : row)
      if (elems(gi) > most) { most = elems(gi); late = gi; }
    for (int gi : row)
      if (gi != late) others += work_of[gi];
    const double slow_pass = 30.0 * most / kSlowPassBytesPerSec;
    if (kProductSlowdown * others / kProductFlopPerSec >= 0.95 * slow_pass && slow_pass >= 1.0e-3) L.late_group = late;
  }
}

void build_layout(const mona_matrix* mats, int count, const mona_options& opt, bool external_state, Layout& L) {
  L.count = count;
  L.external_state = external_state;
  L.ssize = opt.state_dtype == MONA_BF16 ? 2 : 4;
  L.one_buffer = opt.accel_form == MONA_ACCEL_ONE_BUFFER;
  L.caller_slot = opt.accel_form == MONA_ACCEL_CALLER_SLOT;
  size_t off = 0;
  // persistent state, contiguous: this block is what checkpoints carry
  L.state_begin = off;
  L.gprev_off.resize(count);
  L.acc_off.resize(count);
  L.mom_off.resize(count);
  for (int i = 0; i < count; ++i) {
    const size_t ne = (size_t)mats[i].m * mats[i].n;
    L.gprev_off[i] = off;
    if (external_state) { L.acc_off[i] = L.mom_off[i] = off; continue; }
    if (!L.one_buffer && !L.caller_slot) off = align_up(off + ne * L.ssize);
    L.acc_off[i] = off;   off = align_up(off + ne * L.ssize);
    L.mom_off[i] = off;   off = align_up(off + ne * 4);
  }
  L.state_bytes = off - L.state_begin;

  // groups of equal shape (order of first appearance)
  std::map<std::pair<int, int>, int> index;
  L.group_of.resize(count);
  L.rank_in_group.resize(count);
  for (int i = 0; i < count; ++i) {
    auto key = std::make_pair(mats[i].m, mats[i].n);
    auto it = index.find(key);
    int gi;
    if (it == index.end()) {
      gi = (int)L.groups.size();
      index[key] = gi;
      Group g;
      g.m = mats[i].m;
      g.n = mats[i].n;
      g.tall = g.m > g.n;
      const int r128 = round_up(g.m, 128), c128 = round_up(g.n, 128);
      // bf16 rounding errors of the p x p Gram entries average out over p singular directions;
      // below p = 64 they do not, and the products cost nothing there, so they run in fp32
      g.f32 = opt.ns_precision == 1 || std::min(g.m, g.n) <= kSmallSideF32;
      g.esize = g.f32 ? 4 : 2;
      g.gran = (!g.f32 && r128 % 256 == 0 && c128 % 256 == 0) ? 256 : 128;
      g.rows_pad = r128;
      g.cols_pad = c128;
      g.p_pad = g.tall ? g.cols_pad : g.rows_pad;
      // The fused schedule trades products with the long side q for products on the p x p side, so it pays
      // when q is well above p.  Advancing the Gram matrix on the p x p side is as accurate as recomputing
      // it from X while its eigenvalues are still small (the growth phase of the iteration) and less so
      // once they have reached the band around 1.  A full-rank matrix of this shape starts from singular
      // values up to about 1 / sqrt(p) + 1 / sqrt(q) and each early iteration multiplies them by a = 3.4445,
      // so the automatic choice fuses three iterations only where a^2 times that bound is still around one
      // half, and otherwise pairs of iterations, down to a short side of 1024.  Measured O error against the
      // float64 oracle on the benchmark's inputs, (3, 2) / (2, 2, 1) / literal: 1536 x 4096 7.1e-3 / 1.07e-2 /
      // 9.1e-3, 2048 x 8192 6.8e-3 / 1.07e-2 / 9.7e-3; 1024 x 2048 1.5e-2 / 1.2e-2 / 9.5e-3, 1024 x 4096
      // 1.4e-2 / 9.5e-3 / 9.1e-3; 512 x 4096 1.6e-2 / 1.3e-2 / 1.3e-2 (too small to gain: literal).
      const double q_pad = g.tall ? g.rows_pad : g.cols_pad;
      const double start = 1.0 / std::sqrt((double)g.p_pad) + 1.0 / std::sqrt(q_pad);
      g.fused = 0;
      if (!g.f32) {
        if (opt.ns_schedule == MONA_NS_SCHEDULE_FUSED) g.fused = 2;
        else if (opt.ns_schedule == MONA_NS_SCHEDULE_PAIRS) g.fused = 1;
        else if (opt.ns_schedule == MONA_NS_SCHEDULE_AUTO && 2.0 * q_pad >= 3.0 * g.p_pad)
          g.fused = start <= kFusedMaxStart ? 2 : (g.p_pad >= kPairsMinShortSide ? 1 : 0);
      }
      g.npp = g.fused ? 6 : 2;
      L.groups.push_back(g);
    } else {
      gi = it->second;
    }
    L.group_of[i] = gi;
    L.rank_in_group[i] = (int)L.groups[gi].members.size();
    L.groups[gi].members.push_back(i);
  }
  L.work_begin = off;
  for (Group& g : L.groups) {
    const size_t cnt = g.members.size();
    g.x_stride = (int64_t)g.rows_pad * g.cols_pad;
    g.s_stride = (int64_t)g.p_pad * g.p_pad;
    for (int b = 0; b < 2; ++b) { g.x_off[b] = off; off = align_up(off + cnt * g.x_stride * g.esize); }
    for (int b = 0; b < g.npp; ++b) { g.pp_off[b] = off; off = align_up(off + cnt * g.s_stride * g.esize); }
  }
  L.work_bytes = off - L.work_begin;

  plan_lanes(L, opt);

  // elementwise work table
  L.first_block.assign(count, 0);
  L.num_blocks.assign(count, 0);
  for (int pass = 0; pass < 4; ++pass) {
    for (int i = 0; i < count; ++i) {
      if ((mats[i].g_dtype == MONA_BF16) != ((pass & 1) == 1)) continue;
      if ((L.group_of[i] == L.late_group) != (pass >= 2)) continue;
      const int64_t ne = (int64_t)mats[i].m * mats[i].n;
      const int nb = (int)((ne + kEwChunk - 1) / kEwChunk);
      L.first_block[i] = (int)L.blocks.size();
      L.num_blocks[i] = nb;
      for (int c = 0; c < nb; ++c) L.blocks.push_back(BlockWork{i, c});
    }
    L.range_end[pass] = (int)L.blocks.size();
  }
  for (int late = 0; late < 2; ++late) {
    for (int i = 0; i < count; ++i)
      if ((L.group_of[i] == L.late_group) == (late == 1)) L.order.push_back(i);
    if (late == 0) L.num_early = (int)L.order.size();
  }

  // tables
  L.stat_off = off;     off = align_up(off + sizeof(MatStatic) * count);
  L.dyn_off = off;      off = align_up(off + sizeof(MatDynamic) * count);
  L.scales_off = off;   off = align_up(off + sizeof(MatScale) * count);
  L.optr_off = off;     off = align_up(off + sizeof(void*) * count);
  L.order_off = off;    off = align_up(off + sizeof(int32_t) * count);
  L.partials_off = off; off = align_up(off + sizeof(double) * L.blocks.size());
  L.blocks_off = off;   off = align_up(off + sizeof(BlockWork) * L.blocks.size());
  for (Group& g : L.groups) { g.members_off = off; off = align_up(off + sizeof(int32_t) * g.members.size()); }
  L.total = off;
}

struct LaunchRecord {
  int kind, group, iter, tile;
  double flops;
  hipEvent_t e0, e1;
};

}  // namespace

struct mona_state {
  Layout L;
  mona_options opt;
  std::vector<mona_matrix> mats;   // shapes/dtypes given at init (pointers unused)
  char* arena = nullptr;
  int64_t k = 0;
  float last_beta_a = -1.0f;       // one-buffer form: beta_a of the previous step (< 0: none yet)
  // Shape groups are independent of each other, so their Newton-Schulz chains run on separate
  // streams: lane 0 is the caller's stream, lanes 1.. are side streams forked from it after the
  // elementwise pass and joined back before mona_step returns.
  std::vector<hipStream_t> side;       // lanes 1..
  std::vector<hipEvent_t> side_done;   // one per side stream
  hipEvent_t fork_ev = nullptr;
  // the late group's elementwise pass: a stream confined to a quarter of the CUs
  hipStream_t late_stream = nullptr;
  hipEvent_t late_fork = nullptr, late_done = nullptr;
  int late_cus = 0;                    // CUs that stream may use (0: no such stream)
  // pinned ring for the per-step pointer table
  MatDynamic* ring[kRing] = {nullptr, nullptr, nullptr, nullptr};
  hipEvent_t ring_ev[kRing];
  bool ring_used[kRing] = {false, false, false, false};
  int ring_next = 0;
  std::vector<MatDynamic> last_dyn;
  bool dyn_valid = false;
  int device = 0;
  // profiling
  int profiling = 0;
  hipEvent_t ev[kProfSets][4];     // phase marks of the last kProfSets profiled steps, used in turn
  int64_t prof_steps = 0;          // profiled steps since mona_set_profiling
  bool ev_valid = false;
  bool times_ready = false;
  bool fused_update = false;
  bool failed = false;             // a launch failed half way through a step: the state arrays are not usable
  std::vector<LaunchRecord> records;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> event_pool;
  size_t pool_used = 0;

  template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(arena + off); }
};

namespace {

double gemm_flops(const GemmArgs& a) {
  return 2.0 * a.tile_m * a.tile_n * (double)a.K * a.tiles_per_mat * a.count;
}

// One product launch of the plan.
struct Op {
  GemmArgs a;
  int kind = 0;       // OpKind
  int iter = 0;       // Newton-Schulz iteration it belongs to
  TileShape tile{128, 128};
  bool tp = false, tq = false;
};

// Newton-Schulz iterations per chunk.  Literal schedule: one.  Fused schedules: three and then twos, or twos
// only (measured on bf16-rounded products: fusing the late iterations, or more than three of them, loses
// accuracy; three early ones and pairs afterwards do not).
std::vector<int> chunk_sizes(int T, int fused) {
  std::vector<int> out;
  if (!fused) { out.assign(T, 1); return out; }
  int left = T;
  if (fused == 2 && left >= 3) { out.push_back(3); left -= 3; }
  while (left >= 2) { out.push_back(2); left -= 2; }
  if (left) out.push_back(1);
  return out;
}

// Builds the product launches of one group for one step.
//
// Literal schedule, per iteration (Eq. newton_schulz with B = b S + c S S factored out):
//     S = X X^T;  B = b S + c S S;  X <- a X + B X            (tall: S = X^T X, X <- a X + X B)
// Fused schedule, per chunk of n iterations.  With Q_t = a I + b S_t + c S_t^2 one iteration is
// X_{t+1} = Q_t X_t and its Gram matrix is S_{t+1} = Q_t S_t Q_t = S_t Q_t^2 (polynomials of one symmetric
// matrix commute), so n iterations need X only at both ends:
//     S = X X^T;  for i < n:  Q_i = a I + b S + c S S;  (i < n - 1:  U = S Q_i;  S <- U Q_i);  R <- R Q_i  (R_0 = Q_0)
//     X <- R X
// The same polynomial of X in exact arithmetic, with 3 p^2 q + (4 n - 3) p^3 flop instead of n (3 p^2 q + p^3)
// on the symmetric count, i.e. fewer whenever q > p.  Every p x p result is computed on the upper block
// triangle and mirrored.  A chunk of one iteration is the literal iteration.
struct OpBuilder {
  const mona_state* st;
  const Group& g;
  const mona_hparams& hp;
  std::vector<Op>& out;
  int cnt;
  void* X[2];
  void* PP[6];

  OpBuilder(const mona_state* st_, const Group& g_, const mona_hparams& hp_, std::vector<Op>& out_);
  GemmArgs base() const;
  void push(GemmArgs& a, int kind, int iter, bool tp, bool tq, TileShape tile);
  void gram(int src, void* S, bool first, int iter);
  void poly(void* S, void* dst, float diag, int iter);
  void symprod(void* P, void* Q, void* dst, int iter);
  void apply(int src, void* Bm, bool with_e, float beta, bool first, bool last, int iter);
  int build();   // returns the ping-pong buffer that holds O_k afterwards
};

OpBuilder::OpBuilder(const mona_state* st_, const Group& g_, const mona_hparams& hp_, std::vector<Op>& out_)
    : st(st_), g(g_), hp(hp_), out(out_), cnt((int)g_.members.size()) {
  char* base = st->arena;
  for (int b = 0; b < 2; ++b) X[b] = base + g.x_off[b];
  for (int b = 0; b < 6; ++b) PP[b] = b < g.npp ? base + g.pp_off[b] : nullptr;
}

GemmArgs OpBuilder::base() const {
  const Layout& L = st->L;
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.count = cnt;
  a.members = reinterpret_cast<const int32_t*>(st->arena + g.members_off);
  a.scales = st->at<MatScale>(L.scales_off);
  a.stat = st->at<MatStatic>(L.stat_off);
  a.dyn = st->at<MatDynamic>(L.dyn_off);
  a.epilogue = EPI_STORE;
  a.post = POST_NONE;
  return a;
}

void OpBuilder::push(GemmArgs& a, int kind, int iter, bool tp, bool tq, TileShape tile) {
  a.tile_m = tile.bm;
  a.tile_n = tile.bn;
  a.sym_ratio = tile.bm / tile.bn;
  a.tiles_m = a.M / tile.bm;
  a.tiles_n = a.N / tile.bn;
  if (a.symmetric) {
    // row block ti keeps the column blocks from its diagonal on
    a.tiles_per_mat = 0;
    for (int ti = 0; ti < a.tiles_m; ++ti) a.tiles_per_mat += a.tiles_n - a.sym_ratio * ti;
  } else {
    a.tiles_per_mat = a.tiles_m * a.tiles_n;
  }
  Op op;
  op.a = a; op.kind = kind; op.iter = iter; op.tile = tile; op.tp = tp; op.tq = tq;
  out.push_back(op);
}

// The p x p matrices are symmetric bit for bit outside their diagonal tiles (mirrored tiles are copies), and
// inside a diagonal tile either triangle is the product to rounding, so as operands they may be read K-major
// as well as row-major.  The large-tile kernel fetches a K-major operand as 32 contiguous 512-byte rows
// instead of 64-byte pieces of 256 rows and runs 7-13 % faster per K step on it (measured), so it reads them
// that way; the small-tile kernels gain nothing from it.

void OpBuilder::gram(int src, void* S, bool first, int iter) {
  GemmArgs a = base();
  a.P = X[src]; a.Q = X[src]; a.E = nullptr; a.C = S;
  a.strideP = a.strideQ = g.x_stride; a.strideC = g.s_stride;
  a.ldp = a.ldq = g.cols_pad; a.ldc = g.p_pad;
  a.M = a.N = g.p_pad;
  a.K = g.tall ? g.rows_pad : g.cols_pad;
  a.symmetric = 1;
  a.alpha = 1.0f; a.beta = 0.0f;
  if (first) a.post = POST_INV2;
  push(a, OP_GRAM, iter, g.tall, g.tall, pick_tile(g, OP_GRAM, cnt));
}

void OpBuilder::poly(void* S, void* dst, float diag, int iter) {
  const TileShape tile = pick_tile(g, OP_POLY, cnt);
  const bool symk = tile.bm == 256;
  GemmArgs a = base();
  a.P = S; a.Q = S; a.E = S; a.C = dst;
  a.strideP = a.strideQ = a.strideE = a.strideC = g.s_stride;
  a.ldp = a.ldq = a.lde = a.ldc = g.p_pad;
  a.M = a.N = a.K = g.p_pad;
  a.symmetric = 1;
  a.alpha = hp.ns_c; a.beta = hp.ns_b;
  a.diag = diag;
  push(a, OP_POLY, iter, symk, symk, tile);
}

void OpBuilder::symprod(void* P, void* Q, void* dst, int iter) {
  const TileShape tile = pick_tile(g, OP_SYMPROD, cnt);
  const bool symk = tile.bm == 256;
  GemmArgs a = base();
  a.P = P; a.Q = Q; a.E = nullptr; a.C = dst;
  a.strideP = a.strideQ = a.strideC = g.s_stride;
  a.ldp = a.ldq = a.ldc = g.p_pad;
  a.M = a.N = a.K = g.p_pad;
  a.symmetric = 1;
  a.alpha = 1.0f; a.beta = 0.0f;
  push(a, OP_SYMPROD, iter, symk, symk, tile);
}

void OpBuilder::apply(int src, void* Bm, bool with_e, float beta, bool first, bool last, int iter) {
  const TileShape tile = pick_tile(g, OP_APPLY, cnt);
  const bool symk = tile.bm == 256;
  GemmArgs a = base();
  a.E = with_e ? X[src] : nullptr; a.C = X[src ^ 1];
  a.strideE = a.strideC = g.x_stride;
  a.lde = a.ldc = g.cols_pad;
  a.K = g.p_pad;
  a.M = g.rows_pad; a.N = g.cols_pad;
  bool tp, tq;
  if (g.tall) {          // X' = beta X + X B
    a.P = X[src]; a.strideP = g.x_stride; a.ldp = g.cols_pad;
    a.Q = Bm; a.strideQ = g.s_stride; a.ldq = g.p_pad;
    tp = false; tq = symk;
  } else {               // X' = beta X + B X
    a.P = Bm; a.strideP = g.s_stride; a.ldp = g.p_pad;
    a.Q = X[src]; a.strideQ = g.x_stride; a.ldq = g.cols_pad;
    tp = symk && !last;   // the launch that carries the update has no register to spare for a K-major P
    tq = true;
  }
  a.symmetric = 0;
  a.alpha = 1.0f; a.beta = with_e ? beta : 0.0f;
  if (first) a.post = POST_INV;
  if (last) {
    a.epilogue = EPI_UPDATE;
    a.store_out = (hp.flags & MONA_FLAG_KEEP_O) ? 1 : 0;
    a.w_keep = 1.0f - hp.lr * hp.weight_decay;
    a.o_scale = hp.lr * hp.gamma_coeff * sqrtf((float)std::max(g.m, g.n));
  }
  push(a, OP_APPLY, iter, tp, tq, tile);
}

int OpBuilder::build() {
  const int T = hp.ns_steps;
  const std::vector<int> chunks = chunk_sizes(T, g.fused);
  int src = 0, iter = 0;
  for (size_t ci = 0; ci < chunks.size(); ++ci) {
    const int n = chunks[ci];
    const bool first = ci == 0, last = ci + 1 == chunks.size();
    if (n == 1) {
      gram(src, PP[0], first, iter);
      poly(PP[0], PP[1], 0.0f, iter);
      apply(src, PP[1], true, hp.ns_a, first, last, iter);
    } else {
      void* S = PP[0]; void* S2 = PP[1]; void* U = PP[2]; void* Q = PP[3]; void* R = PP[4]; void* R2 = PP[5];
      gram(src, S, first, iter);
      for (int i = 0; i < n; ++i) {
        void* Qi = i == 0 ? R : Q;                 // Q_0 is R_0
        poly(S, Qi, hp.ns_a, iter + i);
        if (i + 1 < n) {
          symprod(S, Qi, U, iter + i);
          symprod(U, Qi, S2, iter + i);
          std::swap(S, S2);
        }
        if (i > 0) {
          symprod(R, Q, R2, iter + i);
          std::swap(R, R2);
        }
      }
      apply(src, R, false, 0.0f, first, last, iter + n - 1);
    }
    src ^= 1;
    iter += n;
  }
  return T == 0 ? 1 : src;
}

// Static description of matrix i: where its state arrays and its working copy live.
void fill_static(const Layout& L, const mona_matrix& q, int i, char* arena, void* g_prev, void* acc, void* mom,
                 MatStatic& ms, void*& o_ptr) {
  const Group& g = L.groups[L.group_of[i]];
  memset(&ms, 0, sizeof ms);
  ms.g_prev = (L.one_buffer || L.caller_slot) ? nullptr : g_prev;
  ms.acc = acc;
  ms.mom = static_cast<float*>(mom);
  ms.x = arena + g.x_off[0] + (size_t)L.rank_in_group[i] * g.x_stride * g.esize;
  ms.m = q.m;
  ms.n = q.n;
  ms.ldx = g.cols_pad;
  ms.w_dtype = q.w_dtype;
  ms.g_dtype = q.g_dtype;
  ms.first_block = L.first_block[i];
  ms.num_blocks = L.num_blocks[i];
  ms.x_f32 = g.f32 ? 1 : 0;
  o_ptr = arena + g.x_off[1] + (size_t)L.rank_in_group[i] * g.x_stride * g.esize;
}

// Theorem 1 assumes |alpha| < 1 / (1 - beta_a).  A step outside that range is taken all the same (the
// algorithm is defined for any alpha); the note is left where mona_last_error() finds it.
void note_unstable_alpha(const mona_hparams* hp) {
  if (hp->flags & MONA_FLAG_MUON_ONLY) return;
  const double bound = 1.0 / (1.0 - (double)hp->beta_a);
  if (std::fabs((double)hp->alpha) >= bound) {
    char buf[256];
    snprintf(buf, sizeof buf, "warning: |alpha| = %g is not below 1 / (1 - beta_a) = %g, the range the convergence "
             "theorem assumes; the step was taken", std::fabs((double)hp->alpha), bound);
    g_err = buf;
  }
}

int check_hparams(const mona_hparams* hp) {
  if (!hp) return fail(MONA_EINVAL, "hparams is NULL");
  if (!(hp->momentum >= 0.0f && hp->momentum < 1.0f)) return fail(MONA_EINVAL, "momentum must lie in [0, 1)");
  if (!(hp->beta_a >= 0.0f && hp->beta_a < 1.0f)) return fail(MONA_EINVAL, "beta_a must lie in [0, 1)");
  if (hp->ns_steps < 0) return fail(MONA_EINVAL, "ns_steps must be >= 0");
  if (!std::isfinite(hp->lr) || !std::isfinite(hp->alpha) || !std::isfinite(hp->weight_decay) ||
      !std::isfinite(hp->ns_a) || !std::isfinite(hp->ns_b) || !std::isfinite(hp->ns_c) ||
      !std::isfinite(hp->gamma_coeff) || !std::isfinite(hp->ns_eps) || hp->ns_eps < 0.0f)
    return fail(MONA_EINVAL, "hyper-parameters must be finite (and ns_eps >= 0)");
  if (hp->flags & ~(MONA_FLAG_FIRST_DIFF_ZERO | MONA_FLAG_KEEP_O | MONA_FLAG_MUON_ONLY)) return fail(MONA_EINVAL, "unknown flag bits");
  return MONA_OK;
}

bool get_event_pair(mona_state* st, hipEvent_t* a, hipEvent_t* b) {
  if (st->pool_used == st->event_pool.size()) {
    hipEvent_t x, y;
    if (hipEventCreate(&x) != hipSuccess) return false;
    if (hipEventCreate(&y) != hipSuccess) { (void)hipEventDestroy(x); return false; }
    st->event_pool.emplace_back(x, y);
  }
  *a = st->event_pool[st->pool_used].first;
  *b = st->event_pool[st->pool_used].second;
  ++st->pool_used;
  return true;
}

}  // namespace

extern "C" {

const char* mona_last_error(void) { return g_err.c_str(); }
const char* mona_version(void) { return "libmona 0.1 (gfx950)"; }

int mona_state_size(const mona_matrix* mats, int32_t count, const mona_options* opts, size_t* bytes_out) {
  if (!bytes_out) return fail(MONA_EINVAL, "bytes_out is NULL");
  int rc = check_mats(mats, count, false);
  if (rc) return rc;
  mona_options o;
  rc = check_opts(opts, &o);
  if (rc) return rc;
  Layout L;
  build_layout(mats, count, o, false, L);
  *bytes_out = L.total;
  return MONA_OK;
}

int mona_init_state(const mona_matrix* mats, int32_t count, const mona_options* opts, void* arena,
                    size_t arena_bytes, void* stream, mona_state** out) {
  if (!out) return fail(MONA_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = check_mats(mats, count, false);
  if (rc) return rc;
  mona_options o;
  rc = check_opts(opts, &o);
  if (rc) return rc;
  if (!arena) return fail(MONA_EINVAL, "arena is NULL");
  if ((uintptr_t)arena % kAlign) return fail(MONA_EINVAL, "arena must be 256-byte aligned");
  mona_state* st = new (std::nothrow) mona_state();
  if (!st) return fail(MONA_ENOMEM, "host allocation failed");
  build_layout(mats, count, o, false, st->L);
  const Layout& L = st->L;
  if (arena_bytes < L.total) {
    const size_t need = L.total;
    delete st;
    return fail(MONA_ENOMEM, "arena too small: %zu bytes given, %zu needed", arena_bytes, need);
  }
  st->opt = o;
  st->mats.assign(mats, mats + count);
  st->arena = static_cast<char*>(arena);
  hipStream_t s = static_cast<hipStream_t>(stream);

  auto cleanup = [&](int code) {
    for (int i = 0; i < kRing; ++i) {
      if (st->ring[i]) { (void)hipHostFree(st->ring[i]); (void)hipEventDestroy(st->ring_ev[i]); }
    }
    if (st->ev_valid)
      for (auto& set : st->ev)
        for (auto& e : set)
          if (e) (void)hipEventDestroy(e);
    for (hipStream_t q : st->side) (void)hipStreamDestroy(q);
    for (hipEvent_t e : st->side_done) (void)hipEventDestroy(e);
    if (st->fork_ev) (void)hipEventDestroy(st->fork_ev);
    if (st->late_stream) (void)hipStreamDestroy(st->late_stream);
    if (st->late_fork) (void)hipEventDestroy(st->late_fork);
    if (st->late_done) (void)hipEventDestroy(st->late_done);
    delete st;
    return code;
  };
#define INIT_TRY(expr)                                                                                   \
  do {                                                                                                   \
    hipError_t e__ = (expr);                                                                             \
    if (e__ != hipSuccess) return cleanup(fail(MONA_EHIP, "%s: %s", #expr, hipGetErrorString(e__)));     \
  } while (0)

  INIT_TRY(hipGetDevice(&st->device));
  for (int i = 0; i < kRing; ++i) {
    void* p = nullptr;
    INIT_TRY(hipHostMalloc(&p, sizeof(MatDynamic) * (size_t)count, hipHostMallocDefault));
    st->ring[i] = static_cast<MatDynamic*>(p);
    hipError_t e = hipEventCreateWithFlags(&st->ring_ev[i], hipEventDisableTiming);
    if (e != hipSuccess) {
      (void)hipHostFree(p);
      st->ring[i] = nullptr;
      return cleanup(fail(MONA_EHIP, "hipEventCreate: %s", hipGetErrorString(e)));
    }
  }
  for (auto& set : st->ev) for (auto& e : set) e = nullptr;
  st->ev_valid = true;             // from here on cleanup() destroys the events created so far
  for (auto& set : st->ev) for (auto& e : set) INIT_TRY(hipEventCreate(&e));
  {
    INIT_TRY(hipEventCreateWithFlags(&st->fork_ev, hipEventDisableTiming));
    for (int i = 1; i < L.lanes; ++i) {
      hipStream_t side = nullptr;
      INIT_TRY(hipStreamCreateWithFlags(&side, hipStreamNonBlocking));
      st->side.push_back(side);
      hipEvent_t done = nullptr;
      INIT_TRY(hipEventCreateWithFlags(&done, hipEventDisableTiming));
      st->side_done.push_back(done);
    }
    if (L.late_group >= 0) {
      // a stream that may use the first quarter of the CUs only (the mask's bits are dealt to the dies in
      // turn, so every die gives up the same number); default priority
      const int cus = device_cu_count();
      const int share = cus / kOverlapCuShare;
      std::vector<uint32_t> mask((cus + 31) / 32, 0u);
      for (int i = 0; i < share; ++i) mask[i / 32] |= 1u << (i % 32);
      INIT_TRY(hipExtStreamCreateWithCUMask(&st->late_stream, (uint32_t)mask.size(), mask.data()));
      INIT_TRY(hipEventCreateWithFlags(&st->late_fork, hipEventDisableTiming));
      INIT_TRY(hipEventCreateWithFlags(&st->late_done, hipEventDisableTiming));
      st->late_cus = share;
    }
  }

  // Alg. 1 initialisation: M_0 = A_0 = G_0 = 0; the padded working copies start (and stay) zero
  INIT_TRY(launch_fill_zero(st->arena + L.state_begin, L.state_bytes + L.work_bytes, s));
  INIT_TRY(launch_fill_zero(st->arena + L.scales_off, align_up(sizeof(MatScale) * count), s));

  std::vector<MatStatic> stat(count);
  std::vector<void*> optr(count);
  for (int i = 0; i < count; ++i) {
    fill_static(L, mats[i], i, st->arena, st->arena + L.gprev_off[i], st->arena + L.acc_off[i],
                st->arena + L.mom_off[i], stat[i], optr[i]);
  }
  INIT_TRY(hipMemcpyAsync(st->arena + L.stat_off, stat.data(), sizeof(MatStatic) * count, hipMemcpyHostToDevice, s));
  INIT_TRY(hipMemcpyAsync(st->arena + L.optr_off, optr.data(), sizeof(void*) * count, hipMemcpyHostToDevice, s));
  INIT_TRY(hipMemcpyAsync(st->arena + L.blocks_off, L.blocks.data(), sizeof(BlockWork) * L.blocks.size(),
                          hipMemcpyHostToDevice, s));
  INIT_TRY(hipMemcpyAsync(st->arena + L.order_off, L.order.data(), sizeof(int32_t) * L.order.size(),
                          hipMemcpyHostToDevice, s));
  for (const Group& g : L.groups) {
    std::vector<int32_t> mem(g.members.begin(), g.members.end());
    INIT_TRY(hipMemcpyAsync(st->arena + g.members_off, mem.data(), sizeof(int32_t) * mem.size(),
                            hipMemcpyHostToDevice, s));
    INIT_TRY(hipStreamSynchronize(s));   // `mem` leaves scope
  }
  INIT_TRY(hipStreamSynchronize(s));     // host vectors above leave scope
#undef INIT_TRY
  *out = st;
  return MONA_OK;
}

}  // extern "C"

namespace {
int step_impl(mona_state* st, const mona_matrix* mats, void* const* slots, int32_t count, const mona_hparams* hp,
              void* stream);
}

extern "C" {

int mona_step(mona_state* st, const mona_matrix* mats, int32_t count, const mona_hparams* hp, void* stream) {
  if (!st) return fail(MONA_EINVAL, "state is NULL");
  if (st->L.caller_slot)
    return fail(MONA_EINVAL, "this state keeps no G_{k-1} (MONA_ACCEL_CALLER_SLOT): use mona_step_streaming");
  return step_impl(st, mats, nullptr, count, hp, stream);
}

int mona_step_streaming(mona_state* st, const mona_matrix* mats, void* const* slots, int32_t count,
                        const mona_hparams* hp, void* stream) {
  if (!st) return fail(MONA_EINVAL, "state is NULL");
  if (!st->L.caller_slot)
    return fail(MONA_EINVAL, "mona_step_streaming needs a state built with MONA_ACCEL_CALLER_SLOT");
  if (!slots) return fail(MONA_EINVAL, "slots is NULL");
  if (count == st->L.count)
    for (int i = 0; i < count; ++i) {
      if (!slots[i]) return fail(MONA_EINVAL, "slot %d is NULL", i);
      if ((uintptr_t)slots[i] & 15) return fail(MONA_EINVAL, "slot %d must be 16-byte aligned", i);
    }
  return step_impl(st, mats, slots, count, hp, stream);
}

}  // extern "C"

namespace {

// Enqueues the kernels of one step (Alg. 1 for every matrix) on `s` and the side streams.  The per-matrix
// tables in the arena must already name this step's w / g pointers.
int enqueue_step(mona_state* st, const mona_hparams* hp, hipStream_t s) {
  Layout& L = st->L;
  const int count = L.count;
  const MatStatic* stat = st->at<MatStatic>(L.stat_off);
  const MatDynamic* dyn = st->at<MatDynamic>(L.dyn_off);
  MatScale* scales = st->at<MatScale>(L.scales_off);
  double* partials = st->at<double>(L.partials_off);
  const BlockWork* blocks = st->at<BlockWork>(L.blocks_off);
  const int nblocks = (int)L.blocks.size();

  // A HIP call that fails once kernels of the step are in flight leaves the state arrays half updated:
  // join whatever was forked, mark the state unusable and say so.
  bool forked = false, late_forked = false;
  auto bail = [&](hipError_t e, const char* what) {
    if (late_forked) {
      (void)hipEventRecord(st->late_done, st->late_stream);
      (void)hipStreamWaitEvent(s, st->late_done, 0);
    }
    if (forked)
      for (size_t i = 0; i < st->side.size(); ++i) {
        (void)hipEventRecord(st->side_done[i], st->side[i]);
        (void)hipStreamWaitEvent(s, st->side_done[i], 0);
      }
    st->failed = true;
    return fail(MONA_EHIP, "%s: %s (the step was abandoned half way: the state arrays are unusable until a checkpoint "
                "is imported with mona_state_import)", what, hipGetErrorString(e));
  };
#define STEP_TRY(expr)                                   \
  do {                                                   \
    hipError_t e__ = (expr);                             \
    if (e__ != hipSuccess) return bail(e__, #expr);      \
  } while (0)

  const bool prof = st->profiling > 0;
  hipEvent_t* const ev = st->ev[st->prof_steps % kProfSets];
  st->times_ready = false;
  st->records.clear();
  st->pool_used = 0;
  if (prof) STEP_TRY(hipEventRecord(ev[0], s));

  // Alg. 1: difference, acceleration EMA, accelerated gradient, momentum, roll; sum of squares.
  // With a late group its pass goes to the stream that owns a quarter of the CUs and runs beside the
  // products of the other groups (not while every launch is timed on its own, and not under stream
  // capture, where the CU mask of a stream would not survive into the graph anyway).
  const bool muon_only = (hp->flags & MONA_FLAG_MUON_ONLY) != 0;
  const int use_prev = muon_only ? 2 : !((hp->flags & MONA_FLAG_FIRST_DIFF_ZERO) && st->k == 0);
  const int sbf = st->opt.state_dtype == MONA_BF16;
  const int one = L.one_buffer ? 1 : 0;
  const int T = hp->ns_steps;
  // (nor on the null stream: a stream with a CU mask can only be created as a blocking one, and the null
  // stream waits for every blocking stream, which would put the two passes in a row again)
  bool overlap = st->late_stream != nullptr && st->profiling < 2 && T > 0 && s != nullptr;
  if (overlap) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    STEP_TRY(hipStreamIsCapturing(s, &cap));
    overlap = cap == hipStreamCaptureStatusNone;
  }
  const int32_t* order = st->at<int32_t>(L.order_off);
  auto pass = [&](int r0, int r1, int g_bf16, hipStream_t q) {
    return launch_state_update(stat, dyn, blocks + r0, partials + r0, r1 - r0, g_bf16, sbf, one, hp->momentum,
                               hp->beta_a, hp->alpha, use_prev, q);
  };
  if (overlap) {
    STEP_TRY(hipEventRecord(st->late_fork, s));
    late_forked = true;
    STEP_TRY(hipStreamWaitEvent(st->late_stream, st->late_fork, 0));
    STEP_TRY(pass(L.range_end[1], L.range_end[2], 0, st->late_stream));
    STEP_TRY(pass(L.range_end[2], L.range_end[3], 1, st->late_stream));
    STEP_TRY(launch_norm_finalize(stat, partials, scales, order + L.num_early, count - L.num_early, hp->ns_eps,
                                  st->late_stream));
    STEP_TRY(hipEventRecord(st->late_done, st->late_stream));
  }
  STEP_TRY(pass(0, L.range_end[0], 0, s));
  STEP_TRY(pass(L.range_end[0], L.range_end[1], 1, s));
  if (!overlap) {
    STEP_TRY(pass(L.range_end[1], L.range_end[2], 0, s));
    STEP_TRY(pass(L.range_end[2], L.range_end[3], 1, s));
  }
  if (L.one_buffer && !muon_only) st->last_beta_a = hp->beta_a;
  STEP_TRY(launch_norm_finalize(stat, partials, scales, order, overlap ? L.num_early : count, hp->ns_eps, s));
  if (prof) STEP_TRY(hipEventRecord(ev[1], s));

  // Newton-Schulz (Eq. newton_schulz), T iterations per shape group
  st->fused_update = T > 0;
  // per-launch timing serialises the launches on the caller's stream so that each interval is one kernel
  const bool fork = !st->side.empty() && st->profiling < 2 && T > 0;
  if (fork) {
    STEP_TRY(hipEventRecord(st->fork_ev, s));
    forked = true;
    for (hipStream_t q : st->side) STEP_TRY(hipStreamWaitEvent(q, st->fork_ev, 0));
  }
  std::vector<Op> ops;
  const int ngroups = (int)L.groups.size();
  for (int pos = 0; pos < ngroups; ++pos) {
    // the late group comes last: its elementwise pass must have finished, and from then on the chip is free
    int gi = pos;
    if (L.late_group >= 0) gi = pos == ngroups - 1 ? L.late_group : (pos < L.late_group ? pos : pos + 1);
    Group& g = L.groups[gi];
    const int lane = fork ? L.lane_of_group[gi] : 0;
    hipStream_t gs = lane == 0 ? s : st->side[lane - 1];
    int cu_cap = 0;
    if (overlap && gi == L.late_group) {
      STEP_TRY(hipStreamWaitEvent(s, st->late_done, 0));
      late_forked = false;
    } else if (overlap) {
      cu_cap = device_cu_count() - st->late_cus;
    }
    ops.clear();
    g.o_buf = OpBuilder(st, g, *hp, ops).build();
    for (const Op& op : ops) {
      LaunchRecord rec;
      const bool each = st->profiling > 1;
      if (each) {
        if (!get_event_pair(st, &rec.e0, &rec.e1)) return bail(hipErrorOutOfMemory, "hipEventCreate");
        STEP_TRY(hipEventRecord(rec.e0, gs));
      }
      STEP_TRY(launch_ns_gemm(op.a, op.tile.bm, op.tp, op.tq, g.f32, cu_cap, gs));
      if (each) {
        STEP_TRY(hipEventRecord(rec.e1, gs));
        rec.kind = op.kind; rec.group = gi; rec.iter = op.iter; rec.tile = op.tile.bm * 1000 + op.tile.bn;
        rec.flops = gemm_flops(op.a);
        st->records.push_back(rec);
      }
    }
  }
  if (fork) {
    for (size_t i = 0; i < st->side.size(); ++i) {
      STEP_TRY(hipEventRecord(st->side_done[i], st->side[i]));
      STEP_TRY(hipStreamWaitEvent(s, st->side_done[i], 0));
    }
    forked = false;
  }
  if (prof) STEP_TRY(hipEventRecord(ev[2], s));
  if (T == 0) {
    // O = X_0, then Eq. muon_update
    STEP_TRY(launch_plain_update(stat, dyn, scales, blocks, nblocks, st->at<void*>(L.optr_off), hp->lr,
                                 hp->weight_decay, hp->gamma_coeff, (hp->flags & MONA_FLAG_KEEP_O) ? 1 : 0, s));
  }
  if (prof) {
    STEP_TRY(hipEventRecord(ev[3], s));
    st->times_ready = true;
    st->prof_steps += 1;
  }
#undef STEP_TRY
  st->k += 1;
  return MONA_OK;
}

int step_impl(mona_state* st, const mona_matrix* mats, void* const* slots, int32_t count, const mona_hparams* hp,
              void* stream) {
  g_err.clear();
  if (st->failed)
    return fail(MONA_EHIP, "this state was left half updated by a failed launch in an earlier step: import a "
                "checkpoint with mona_state_import first");
  int rc = check_mats(mats, count, true);
  if (rc) return rc;
  rc = check_hparams(hp);
  if (rc) return rc;
  const Layout& L = st->L;
  if (count != L.count) return fail(MONA_ESHAPE, "count %d differs from %d at init", count, L.count);
  for (int i = 0; i < count; ++i) {
    const mona_matrix& a = mats[i];
    const mona_matrix& b = st->mats[i];
    if (a.m != b.m || a.n != b.n || a.w_dtype != b.w_dtype || a.g_dtype != b.g_dtype)
      return fail(MONA_ESHAPE, "matrix %d: shape or dtype differs from init (%d x %d vs %d x %d)", i, a.m, a.n, b.m,
                  b.n);
  }
  const bool muon_only = (hp->flags & MONA_FLAG_MUON_ONLY) != 0;
  if (L.one_buffer && !muon_only) {
    // C_{k+1} was formed with the previous step's beta_a: the identity A_k = C_k + (1 - beta_a) G_k
    // holds only if this step uses the same value
    if (st->last_beta_a >= 0.0f && st->last_beta_a != hp->beta_a)
      return fail(MONA_EINVAL, "one-buffer form: beta_a changed from %g to %g between steps", (double)st->last_beta_a,
                  (double)hp->beta_a);
  }
  hipStream_t s = static_cast<hipStream_t>(stream);

  // per-step pointer table
  bool changed = !st->dyn_valid;
  if (!changed)
    for (int i = 0; i < count; ++i)
      if (st->last_dyn[i].w != mats[i].w || st->last_dyn[i].g != mats[i].g ||
          st->last_dyn[i].slot != (slots ? slots[i] : nullptr)) { changed = true; break; }
  if (changed) {
    const int slot = st->ring_next;
    if (st->ring_used[slot]) HIP_TRY(hipEventSynchronize(st->ring_ev[slot]));
    st->last_dyn.resize(count);
    for (int i = 0; i < count; ++i) {
      st->last_dyn[i].w = mats[i].w;
      st->last_dyn[i].g = mats[i].g;
      st->last_dyn[i].slot = slots ? slots[i] : nullptr;
      st->ring[slot][i] = st->last_dyn[i];
    }
    HIP_TRY(hipMemcpyAsync(st->arena + L.dyn_off, st->ring[slot], sizeof(MatDynamic) * count, hipMemcpyHostToDevice,
                           s));
    HIP_TRY(hipEventRecord(st->ring_ev[slot], s));
    st->ring_used[slot] = true;
    st->ring_next = (slot + 1) % kRing;
    st->dyn_valid = true;
  }
  rc = enqueue_step(st, hp, s);
  if (rc) return rc;
  note_unstable_alpha(hp);
  return MONA_OK;
}

}  // namespace

// ---- the entry point that allocates nothing -------------------------------------------------------------
namespace {

// Workspace of mona_step_noalloc: what mona_step keeps in the caller's arena beyond the state arrays (the
// working copies X, the p x p matrices, per-block partial sums, scales and the small tables), here in a
// static device array.  Every GPU the library runs on holds its own copy, at its own address, until the
// process ends.
constexpr size_t kScratchBytes = MONA_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, looked up once

// Device address of the scratch array on the current device.  In host code the array's name is only a
// handle for this lookup, never an address to hand to a kernel.
int scratch_on_current_device(char** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(MONA_EUNSUPPORTED, "device ordinal %d is beyond %d", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(MONA_EHIP, "hipGetSymbolAddress returned a null address for the scratch array");
    g_scratch_ptr[dev] = p;
  }
  *out = static_cast<char*>(g_scratch_ptr[dev]);
  return MONA_OK;
}

}  // namespace

extern "C" {

int mona_step_noalloc(const mona_matrix* mat, const mona_options* opts, void* g_prev, void* acc, void* mom,
                      const mona_hparams* hp, int64_t k, void* stream) {
  g_err.clear();
  int rc = check_mats(mat, 1, true);
  if (rc) return rc;
  rc = check_hparams(hp);
  if (rc) return rc;
  mona_options o;
  rc = check_opts(opts, &o);
  if (rc) return rc;
  if (o.accel_form != MONA_ACCEL_TWO_BUFFER)
    return fail(MONA_EUNSUPPORTED, "mona_step_noalloc takes the state arrays of Alg. 1 (MONA_ACCEL_TWO_BUFFER) only");
  if (k < 0) return fail(MONA_EINVAL, "k must be >= 0");
  if (!g_prev || !acc || !mom) return fail(MONA_EINVAL, "g_prev, acc and mom must not be NULL");
  if (((uintptr_t)g_prev & 15) || ((uintptr_t)acc & 15) || ((uintptr_t)mom & 15))
    return fail(MONA_EINVAL, "g_prev, acc and mom must be 16-byte aligned");
  // the same plan a one-matrix mona_init_state would build, laid out over the scratch array
  mona_state st;
  build_layout(mat, 1, o, true, st.L);
  const Layout& L = st.L;
  if (L.total > kScratchBytes)
    return fail(MONA_ENOMEM, "a %d x %d matrix needs %zu bytes of workspace; the static scratch of mona_step_noalloc "
                "holds %zu (use mona_step with an arena for larger matrices)", mat->m, mat->n, L.total, kScratchBytes);
  char* base = nullptr;
  rc = scratch_on_current_device(&base);
  if (rc) return rc;
  st.opt = o;
  st.mats.assign(mat, mat + 1);
  st.arena = base;
  st.k = k;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // The array keeps what the last call left in it: the padding of the working matrices and the scales must
  // start from zero (a fill kernel, not a memset: the call may be under graph capture).
  HIP_TRY(launch_fill_zero(base + L.work_begin, L.work_bytes, s));
  HIP_TRY(launch_fill_zero(base + L.scales_off, align_up(sizeof(MatScale)), s));
  MatStatic ms;
  void* o_ptr = nullptr;
  fill_static(L, *mat, 0, base, g_prev, acc, mom, ms, o_ptr);
  MatDynamic md;
  md.w = mat->w; md.g = mat->g; md.slot = nullptr;
  HIP_TRY(launch_single_tables(ms, md, o_ptr, st.at<MatStatic>(L.stat_off), st.at<MatDynamic>(L.dyn_off),
                               st.at<void*>(L.optr_off), st.at<BlockWork>(L.blocks_off), (int)L.blocks.size(),
                               reinterpret_cast<int32_t*>(base + L.groups[0].members_off),
                               st.at<int32_t>(L.order_off), s));
  rc = enqueue_step(&st, hp, s);
  if (rc) return rc;
  note_unstable_alpha(hp);
  return MONA_OK;
}

}  // extern "C"

extern "C" {

int mona_free_state(mona_state* st) {
  if (!st) return MONA_OK;
  for (int i = 0; i < kRing; ++i) {
    if (st->ring_used[i]) (void)hipEventSynchronize(st->ring_ev[i]);
    if (st->ring[i]) { (void)hipHostFree(st->ring[i]); (void)hipEventDestroy(st->ring_ev[i]); }
  }
  if (st->ev_valid)
    for (auto& set : st->ev)
      for (auto& e : set)
        if (e) (void)hipEventDestroy(e);
  for (auto& pr : st->event_pool) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
  for (hipStream_t q : st->side) { (void)hipStreamSynchronize(q); (void)hipStreamDestroy(q); }
  for (hipEvent_t e : st->side_done) (void)hipEventDestroy(e);
  if (st->fork_ev) (void)hipEventDestroy(st->fork_ev);
  if (st->late_stream) { (void)hipStreamSynchronize(st->late_stream); (void)hipStreamDestroy(st->late_stream); }
  if (st->late_fork) (void)hipEventDestroy(st->late_fork);
  if (st->late_done) (void)hipEventDestroy(st->late_done);
  delete st;
  return MONA_OK;
}

int mona_state_view(mona_state* st, int32_t i, int32_t kind, mona_view* out) {
  if (!st || !out) return fail(MONA_EINVAL, "state or out is NULL");
  const Layout& L = st->L;
  if (i < 0 || i >= L.count) return fail(MONA_EINVAL, "matrix index %d out of range [0, %d)", i, L.count);
  const mona_matrix& q = st->mats[i];
  const Group& g = L.groups[L.group_of[i]];
  out->rows = q.m; out->cols = q.n; out->ld = q.n;
  switch (kind) {
    case MONA_VIEW_G_PREV:
      if (L.one_buffer) return fail(MONA_EUNSUPPORTED, "the one-buffer form stores no G_{k-1}");
      if (L.caller_slot) return fail(MONA_EUNSUPPORTED, "G_{k-1} is kept by the caller (MONA_ACCEL_CALLER_SLOT)");
      out->ptr = st->arena + L.gprev_off[i]; out->dtype = st->opt.state_dtype; break;
    case MONA_VIEW_A:
      if (L.one_buffer) return fail(MONA_EUNSUPPORTED, "the one-buffer form stores C, not A (use MONA_VIEW_C)");
      out->ptr = st->arena + L.acc_off[i]; out->dtype = st->opt.state_dtype; break;
    case MONA_VIEW_C:
      if (!L.one_buffer) return fail(MONA_EUNSUPPORTED, "MONA_VIEW_C exists only in the one-buffer form");
      out->ptr = st->arena + L.acc_off[i]; out->dtype = st->opt.state_dtype; break;
    case MONA_VIEW_M: out->ptr = st->arena + L.mom_off[i]; out->dtype = MONA_F32; break;
    case MONA_VIEW_NORM:
      out->ptr = reinterpret_cast<char*>(st->at<MatScale>(L.scales_off) + i) + offsetof(MatScale, norm);
      out->rows = out->cols = out->ld = 1; out->dtype = MONA_F32;
      break;
    case MONA_VIEW_O: {
      // every chunk of iterations reads one ping-pong buffer and writes the other; with T = 0 the update
      // kernel writes buffer 1
      out->ptr = st->arena + g.x_off[g.o_buf] + (size_t)L.rank_in_group[i] * g.x_stride * g.esize;
      out->ld = g.cols_pad;
      out->dtype = g.f32 ? MONA_F32 : MONA_BF16;
      break;
    }
    default: return fail(MONA_EINVAL, "unknown view kind %d", kind);
  }
  return MONA_OK;
}

int mona_state_export_size(mona_state* st, size_t* bytes_out) {
  if (!st || !bytes_out) return fail(MONA_EINVAL, "state or bytes_out is NULL");
  *bytes_out = st->L.state_bytes;
  return MONA_OK;
}

int mona_state_export(mona_state* st, void* dst, size_t dst_bytes, void* stream) {
  if (!st || !dst) return fail(MONA_EINVAL, "state or dst is NULL");
  if (dst_bytes < st->L.state_bytes) return fail(MONA_ENOMEM, "dst too small: %zu < %zu", dst_bytes, st->L.state_bytes);
  HIP_TRY(hipMemcpyAsync(dst, st->arena + st->L.state_begin, st->L.state_bytes, hipMemcpyDeviceToDevice,
                         static_cast<hipStream_t>(stream)));
  return MONA_OK;
}

int mona_state_import(mona_state* st, const void* src, size_t src_bytes, int64_t step_count, void* stream) {
  if (!st || !src) return fail(MONA_EINVAL, "state or src is NULL");
  if (src_bytes != st->L.state_bytes)
    return fail(MONA_ESHAPE, "checkpoint holds %zu bytes, this state needs %zu", src_bytes, st->L.state_bytes);
  if (step_count < 0) return fail(MONA_EINVAL, "step_count must be >= 0");
  HIP_TRY(hipMemcpyAsync(st->arena + st->L.state_begin, src, st->L.state_bytes, hipMemcpyDeviceToDevice,
                         static_cast<hipStream_t>(stream)));
  // The products rely on the padding of the working matrices being zero.  The steps themselves keep it so;
  // clearing it here as well makes an imported state independent of whatever the arena went through before.
  HIP_TRY(launch_fill_zero(st->arena + st->L.work_begin, st->L.work_bytes, static_cast<hipStream_t>(stream)));
  st->failed = false;
  st->k = step_count;
  st->last_beta_a = -1.0f;   // the checkpoint does not say which beta_a formed C
  return MONA_OK;
}

int mona_state_step_count(mona_state* st, int64_t* k_out) {
  if (!st || !k_out) return fail(MONA_EINVAL, "state or k_out is NULL");
  *k_out = st->k;
  return MONA_OK;
}

int mona_state_status(mona_state* st, uint32_t* host_out, int32_t count, void* stream) {
  if (!st || !host_out) return fail(MONA_EINVAL, "state or host_out is NULL");
  if (count != st->L.count) return fail(MONA_ESHAPE, "count %d differs from %d at init", count, st->L.count);
  std::vector<MatScale> tmp(count);
  hipStream_t s = static_cast<hipStream_t>(stream);
  HIP_TRY(hipMemcpyAsync(tmp.data(), st->arena + st->L.scales_off, sizeof(MatScale) * count, hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  for (int i = 0; i < count; ++i) host_out[i] = tmp[i].status;
  return MONA_OK;
}

int mona_set_profiling(mona_state* st, int32_t on) {
  if (!st) return fail(MONA_EINVAL, "state is NULL");
  if (on < 0 || on > 2) return fail(MONA_EINVAL, "profiling level must be 0, 1 or 2");
  st->profiling = on;
  st->times_ready = false;
  st->prof_steps = 0;
  return MONA_OK;
}

int mona_last_step_times(mona_state* st, float* ms_out) {
  if (!st || !ms_out) return fail(MONA_EINVAL, "state or ms_out is NULL");
  if (!st->times_ready) return fail(MONA_EINVAL, "no profiled step yet (call mona_set_profiling(st, 1) first)");
  hipEvent_t* const ev = st->ev[(st->prof_steps - 1) % kProfSets];
  HIP_TRY(hipEventSynchronize(ev[3]));
  HIP_TRY(hipEventElapsedTime(&ms_out[0], ev[0], ev[1]));
  HIP_TRY(hipEventElapsedTime(&ms_out[1], ev[1], ev[2]));
  HIP_TRY(hipEventElapsedTime(&ms_out[2], ev[2], ev[3]));
  HIP_TRY(hipEventElapsedTime(&ms_out[3], ev[0], ev[3]));
  return MONA_OK;
}

int mona_mean_step_times(mona_state* st, float* ms_out, int32_t* steps_out) {
  if (!st || !ms_out || !steps_out) return fail(MONA_EINVAL, "state, ms_out or steps_out is NULL");
  if (!st->times_ready) return fail(MONA_EINVAL, "no profiled step yet (call mona_set_profiling(st, 1) first)");
  const int n = (int)std::min<int64_t>(st->prof_steps, kProfSets);
  double sum[4] = {0.0, 0.0, 0.0, 0.0};
  for (int b = 0; b < n; ++b) {
    hipEvent_t* const ev = st->ev[(st->prof_steps - 1 - b) % kProfSets];
    HIP_TRY(hipEventSynchronize(ev[3]));
    const int from[4] = {0, 1, 2, 0}, to[4] = {1, 2, 3, 3};
    for (int i = 0; i < 4; ++i) {
      float ms = 0.0f;
      HIP_TRY(hipEventElapsedTime(&ms, ev[from[i]], ev[to[i]]));
      sum[i] += ms;
    }
  }
  for (int i = 0; i < 4; ++i) ms_out[i] = (float)(sum[i] / n);
  *steps_out = n;
  return MONA_OK;
}

int mona_last_step_launches(mona_state* st, mona_launch_time* out, int32_t max_records, int32_t* n_out) {
  if (!st || !n_out) return fail(MONA_EINVAL, "state or n_out is NULL");
  if (st->profiling < 2 || !st->times_ready) return fail(MONA_EINVAL, "no step profiled at level 2 yet");
  HIP_TRY(hipEventSynchronize(st->ev[(st->prof_steps - 1) % kProfSets][3]));
  const int n = (int)st->records.size();
  *n_out = n;
  if (!out) return MONA_OK;
  for (int i = 0; i < n && i < max_records; ++i) {
    const LaunchRecord& r = st->records[i];
    out[i].kind = r.kind; out[i].group = r.group; out[i].iter = r.iter; out[i].tile = r.tile;
    out[i].flops = r.flops;
    const Group& g = st->L.groups[r.group];
    out[i].m = g.m; out[i].n = g.n; out[i].count = (int)g.members.size();
    HIP_TRY(hipEventElapsedTime(&out[i].ms, r.e0, r.e1));
  }
  return MONA_OK;
}

int mona_plan_info(mona_state* st, int32_t ns_steps, int64_t* launches_out, double* ns_flops_executed_out,
                   double* elementwise_bytes_out) {
  if (!st) return fail(MONA_EINVAL, "state is NULL");
  if (ns_steps < 0) return fail(MONA_EINVAL, "ns_steps must be >= 0");
  const Layout& L = st->L;
  mona_hparams hp;
  memset(&hp, 0, sizeof hp);
  hp.ns_steps = ns_steps;
  double flops = 0.0;
  int64_t launches = 0;
  std::vector<Op> ops;
  for (const Group& g : L.groups) {
    ops.clear();
    OpBuilder(st, g, hp, ops).build();
    for (const Op& op : ops) flops += gemm_flops(op.a);
    launches += (int64_t)ops.size();
  }
  double bytes = 0.0;
  for (int i = 0; i < L.count; ++i) {
    const double ne = (double)st->mats[i].m * st->mats[i].n;
    const double gsz = st->mats[i].g_dtype == MONA_BF16 ? 2 : 4;
    // state pass: read G, G_prev, A, M; write G_prev, A, M and the working copy of M
    // (one-buffer form: C in place of G_prev and A)
    const double aux = (L.one_buffer ? 1 : 2) * L.ssize;
    bytes += ne * (gsz + aux + 4 + aux + 4 + L.groups[L.group_of[i]].esize);
  }
  if (launches_out) *launches_out = launches;
  if (ns_flops_executed_out) *ns_flops_executed_out = flops;
  if (elementwise_bytes_out) *elementwise_bytes_out = bytes;
  return MONA_OK;
}

}  // extern "C"
