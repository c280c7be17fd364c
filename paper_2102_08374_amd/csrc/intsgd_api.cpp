// Host side of the C ABI declared in include/intsgd.h: argument validation (always
// before anything touches the device), the tiling plan and its per-partition device
// table, workspace carving, and the sequencing of kernel launches.

#include <hip/hip_runtime_api.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <list>
#include <mutex>
#include <string>
#include <vector>

#include "intsgd.h"
#include "intsgd_internal.h"

namespace intsgd {
namespace {

constexpr uint32_t kMinTile = 1024;
constexpr uint32_t kMaxTile = 65536;
constexpr uint32_t kMaxGrid = 1u << 20;
constexpr uint64_t kMaxD = 1ull << 40;
constexpr size_t kAlign = 256;
constexpr uint32_t kLdsPerCu = 160u * 1024u;    // gfx950

// The caller's launch options (a zero field means "automatic"), copied once per call so
// that a call sees one consistent set even if the caller's struct changes under it.
struct Tuning {
  uint32_t tile_coords, max_workgroups, workgroups_per_cu, two_phase;
};

Tuning requested_tuning(const intsgd_desc* desc) {
  const intsgd_launch_opts* o = desc->launch;
  if (o == nullptr) return Tuning{0, 0, 0, 0};
  return Tuning{o->tile_coords, o->max_workgroups, o->workgroups_per_cu, o->two_phase};
}

// Automatic choices of the tile sweeps, measured on MI355X: 8 KB per stream and workgroup (one
// quad per thread) in both rounding modes, and as few resident workgroups as keep enough loads
// in flight: two of 512 threads per CU when a thread has two groups of eight worker loads to
// issue (n > 8), four when it has at most one (at n = 8: 82 % of peak against 76 %).
// Randomized rounding: the reservation is for four, of which the kernel's 75 VGPRs let three be
// resident; with its per-coordinate clamp and clip test gone (fast path) it no longer gains
// from 16 KB tiles (8 KB: 1-2.5 % faster on 8 x 25.6 M, 8 x 108 M and 8 x 1.3 B).
Tuning effective_tuning(const intsgd_desc* desc) {
  const bool random = desc->rounding == INTSGD_ROUND_STOCHASTIC;
  Tuning t = requested_tuning(desc);
  if (t.tile_coords == 0) t.tile_coords = 2048;
  if (t.max_workgroups == 0) t.max_workgroups = kMaxGrid;
  if (t.workgroups_per_cu == 0) t.workgroups_per_cu = (random || desc->n <= 8) ? 4 : 2;
  return t;
}

// The two-phase sweep needs one block and enough coordinates to give every CU a chunk.  It is
// never the automatic choice: with the XCD-aware tile order and a tile sized by the worker
// count the tile sweep streams as fast or faster for every n measured (nearest-even, d = 25.6 M
// and 108 M; n = 1: 75-81 % of peak against 69-75 %, n = 2: 81-83 % against 77-81 %, n = 5:
// 84-85 % against 80-81 %, n = 8: 87-89 % against 83 %, n = 16: 87 % against 85 %; n = 4 at
// 108 M is the one tie), and randomized rounding fills the read phase with arithmetic anyway.
// Callers ask for it with two_phase = 2.
constexpr uint64_t kMinPhasedD = 1ull << 22;
// Consecutive workgroups go to the 8 XCDs in turn.  The sweeps that read the gradient streams run
// faster when each XCD takes runs of 16 consecutive tiles instead of every eighth tile: a1-a3 by
// 3 % (108 M coordinates) to 10 % (1.3 G), F1, the momentum form, IntDIANA and the nearest-even
// fused sweep by 1-3 %.  The randomized fused sweep gains 1.5-2 % at 635 K tiles, 1 % at 53 K and
// nothing at 12 K (-0.3 %); the decode kernels are slower with runs at any size.
constexpr uint32_t kXcdRunFromTiles = 1u << 10;
constexpr uint32_t kXcdRunFromTilesRandomFused = 1u << 15;
constexpr uint32_t kXcdRunShift = 4;
bool use_two_phase(const intsgd_desc* desc, const Tuning& t) {
  if (desc->num_blocks != 1 || desc->d < kMinPhasedD || t.two_phase == 1) return false;
  if (t.two_phase == 2) return true;
  return false;
}

thread_local std::string t_hip_error;

// The profiling events of the caller's launch options (if any) go to the call's streaming kernel.
void take_taps(const intsgd_desc* desc, LaunchShape* ls) {
  const intsgd_launch_opts* o = desc->launch;
  ls->tap_start = o ? static_cast<hipEvent_t>(o->start_event) : nullptr;
  ls->tap_stop = o ? static_cast<hipEvent_t>(o->stop_event) : nullptr;
}

intsgd_status hip_fail(hipError_t e) {
  t_hip_error = std::string(hipGetErrorName(e)) + ": " + hipGetErrorString(e);
  return INTSGD_EHIP;
}

// Compute units of the current device (cached per device id).
intsgd_status compute_units(uint32_t* out) {
  static std::mutex m;
  static std::vector<int> cache;
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return hip_fail(e);
  std::lock_guard<std::mutex> lock(m);
  if ((size_t)device >= cache.size()) cache.resize(device + 1, 0);
  if (cache[device] == 0) {
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
    if (e != hipSuccess) return hip_fail(e);
    cache[device] = cus > 0 ? cus : 1;
  }
  *out = (uint32_t)cache[device];
  return INTSGD_OK;
}

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

intsgd_status validate_launch_opts(const intsgd_launch_opts* o) {
  if (o == nullptr) return INTSGD_OK;
  const uint32_t tile = o->tile_coords, grid = o->max_workgroups, wgs = o->workgroups_per_cu;
  if (tile != 0 && (tile < kMinTile || tile > kMaxTile || tile % kMinTile != 0)) return INTSGD_EINVAL;
  if (grid > kMaxGrid) return INTSGD_EINVAL;
  if (wgs != 0 && (wgs < 2 || wgs > 8)) return INTSGD_EINVAL;
  if (o->two_phase > 2) return INTSGD_EINVAL;
  if ((o->start_event == nullptr) != (o->stop_event == nullptr)) return INTSGD_EINVAL;
  return INTSGD_OK;
}

intsgd_status validate_desc(const intsgd_desc* desc) {
  if (desc == nullptr) return INTSGD_EINVAL;
  if (desc->d == 0 || desc->n == 0 || desc->num_blocks == 0) return INTSGD_EINVAL;
  if (desc->d > kMaxD) return INTSGD_ERANGE;
  if (desc->n > INTSGD_MAX_WORKERS) return INTSGD_ERANGE;
  if (desc->num_blocks > desc->d) return INTSGD_EINVAL;
  if (desc->rounding != INTSGD_ROUND_NEAREST_EVEN && desc->rounding != INTSGD_ROUND_STOCHASTIC)
    return INTSGD_EINVAL;
  if (desc->wire != INTSGD_WIRE_INT8 && desc->wire != INTSGD_WIRE_INT32) return INTSGD_EINVAL;
  if (desc->clip < 1) return INTSGD_ERANGE;
  if ((int64_t)desc->n * (int64_t)desc->clip > (int64_t)INT32_MAX) return INTSGD_ERANGE;
  if (desc->wire == INTSGD_WIRE_INT8 && desc->clip > 127) return INTSGD_ERANGE;
  if (desc->num_blocks > 1 || desc->block_offsets != nullptr) {
    const uint64_t* off = desc->block_offsets;
    if (off == nullptr) return INTSGD_EINVAL;
    if (off[0] != 0 || off[desc->num_blocks] != desc->d) return INTSGD_EINVAL;
    for (uint32_t l = 0; l < desc->num_blocks; ++l)
      if (off[l + 1] <= off[l]) return INTSGD_EINVAL;
  }
  if ((reinterpret_cast<uintptr_t>(desc->largest_sum) & 3u) != 0) return INTSGD_EALIGN;
  return validate_launch_opts(desc->launch);
}

intsgd_status validate_rule(double beta, double eps, double eta) {
  if (!(beta >= 0.0 && beta < 1.0)) return INTSGD_EINVAL;
  if (!(eps >= 0.0) || !std::isfinite(eps)) return INTSGD_EINVAL;
  if (!(eta > 0.0) || !std::isfinite(eta)) return INTSGD_EINVAL;
  return INTSGD_OK;
}

intsgd_status validate_worker_ptrs(const void* const* ptrs, uint32_t n) {
  if (ptrs == nullptr) return INTSGD_EINVAL;
  for (uint32_t i = 0; i < n; ++i) {
    if (ptrs[i] == nullptr) return INTSGD_EINVAL;
    if (!aligned16(ptrs[i])) return INTSGD_EALIGN;
  }
  return INTSGD_OK;
}

intsgd_status validate_vec(const void* p) {
  if (p == nullptr) return INTSGD_EINVAL;
  if (!aligned16(p)) return INTSGD_EALIGN;
  return INTSGD_OK;
}

uint64_t tiles_of(uint64_t len, uint32_t tile) { return (len + tile - 1) / tile; }

// Workspace carving: [norm partial per tile][first-level norm sums][clip hint]
// [clip flag per workgroup][clip counts per workgroup and worker]; sized for the
// smallest tile so that it is valid under any tuning (the grid never exceeds the
// number of tiles).
struct WorkspaceLayout {
  size_t norm_off, mid_off, hint_off, any_off, rows_off, big_off, bigmid_off, total;
};

// Layout for at most max_tiles work tiles (or workgroups, whichever is larger).
WorkspaceLayout workspace_layout_for(const intsgd_desc* desc, uint64_t max_tiles) {
  WorkspaceLayout w;
  w.norm_off = 0;
  w.mid_off = w.norm_off + round_up((size_t)max_tiles * sizeof(double), kAlign);
  w.hint_off = w.mid_off + round_up((size_t)(max_tiles / 4096 + 2) * sizeof(double), kAlign);
  w.any_off = w.hint_off + kAlign;
  w.rows_off = w.any_off + round_up((size_t)max_tiles * sizeof(uint32_t), kAlign);
  w.big_off = w.rows_off + round_up((size_t)max_tiles * desc->n * sizeof(uint64_t), kAlign);
  w.bigmid_off = w.big_off + round_up((size_t)max_tiles * sizeof(uint32_t), kAlign);
  w.total = w.bigmid_off + round_up((size_t)(max_tiles / 4096 + 2) * sizeof(uint32_t), kAlign);
  return w;
}

// The caller-owned workspace: sized for the smallest tile, so valid under any launch options.
WorkspaceLayout workspace_layout(const intsgd_desc* desc) {
  return workspace_layout_for(desc, tiles_of(desc->d, kMinTile) + desc->num_blocks);
}

intsgd_status validate_workspace(const intsgd_desc* desc, void* ws, size_t bytes) {
  if (ws == nullptr) return INTSGD_EWORKSPACE;
  if ((reinterpret_cast<uintptr_t>(ws) & (kAlign - 1)) != 0) return INTSGD_EWORKSPACE;
  if (bytes < workspace_layout(desc).total) return INTSGD_EWORKSPACE;
  return INTSGD_OK;
}

template <class T>
T* ws_at(void* ws, size_t off) {
  return reinterpret_cast<T*>(static_cast<char*>(ws) + off);
}

RoundSpec round_spec(const intsgd_desc* desc) {
  RoundSpec rs;
  rs.rounding = desc->rounding;
  rs.clip = desc->clip;
  // smallest fp32 that is >= L+1 (L+1 itself need not be an fp32 number)
  const double bound = (double)desc->clip + 1.0;
  float thr = (float)bound;
  if ((double)thr < bound) thr = std::nextafterf(thr, INFINITY);
  rs.sat_threshold = thr;
  // largest fp32 <= L (L >= 1): a scaled value below it in magnitude rounds into [-L, L] either way
  float lim = (float)desc->clip;
  if ((double)lim > (double)desc->clip) lim = std::nextafterf(lim, 0.0f);
  std::memcpy(&rs.fast_limit_bits, &lim, sizeof(lim));
  rs.key0 = (uint32_t)desc->seed;
  rs.key1 = (uint32_t)(desc->seed >> 32);
  rs.step = desc->step;
  return rs;
}

// ---------------------------------------------------------------- per-partition device table
struct DevicePlan {
  int device;
  uint32_t tile;
  uint64_t d;
  std::vector<uint64_t> offsets;
  uint32_t num_tiles;
  TileEntry* table;        // device
  uint32_t* tile_prefix;   // device, B+1
  uint64_t* offsets_dev;   // device, B+1
};

std::mutex g_mutex;
std::list<DevicePlan> g_plans;   // stable addresses: callers hold a pointer during their call

void free_plan(DevicePlan& p) {
  int cur = 0;
  const bool have_cur = hipGetDevice(&cur) == hipSuccess;
  if (hipSetDevice(p.device) == hipSuccess) {
    (void)hipFree(p.table);
    (void)hipFree(p.tile_prefix);
    (void)hipFree(p.offsets_dev);
  }
  if (have_cur) (void)hipSetDevice(cur);
}

// Looks up or (if may_build) builds the device table of a multi-block partition.
intsgd_status get_plan(const intsgd_desc* desc, uint32_t tile, const DevicePlan** out,
                       bool may_build = true) {
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return hip_fail(e);
  const uint32_t B = desc->num_blocks;
  std::lock_guard<std::mutex> lock(g_mutex);
  for (const DevicePlan& p : g_plans) {
    if (p.device == device && p.tile == tile && p.d == desc->d && p.offsets.size() == B + 1 &&
        std::memcmp(p.offsets.data(), desc->block_offsets, (B + 1) * sizeof(uint64_t)) == 0) {
      *out = &p;
      return INTSGD_OK;
    }
  }
  if (!may_build) return INTSGD_ENOPLAN;
  std::vector<TileEntry> table;
  std::vector<uint32_t> prefix(B + 1);
  for (uint32_t l = 0; l < B; ++l) {
    prefix[l] = (uint32_t)table.size();
    const uint64_t s = desc->block_offsets[l], e2 = desc->block_offsets[l + 1];
    for (uint64_t pos = s; pos < e2; pos += tile) {
      const uint64_t len = (e2 - pos < tile) ? (e2 - pos) : tile;
      table.push_back(TileEntry{pos, (uint32_t)len, l});
    }
  }
  prefix[B] = (uint32_t)table.size();
  DevicePlan p{};
  p.device = device;
  p.tile = tile;
  p.d = desc->d;
  p.offsets.assign(desc->block_offsets, desc->block_offsets + B + 1);
  p.num_tiles = (uint32_t)table.size();
  const size_t tb = table.size() * sizeof(TileEntry), pb = prefix.size() * sizeof(uint32_t),
               ob = p.offsets.size() * sizeof(uint64_t);
  e = hipMalloc((void**)&p.table, tb);
  if (e == hipSuccess) e = hipMalloc((void**)&p.tile_prefix, pb);
  if (e == hipSuccess) e = hipMalloc((void**)&p.offsets_dev, ob);
  if (e == hipSuccess) e = hipMemcpy(p.table, table.data(), tb, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(p.tile_prefix, prefix.data(), pb, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(p.offsets_dev, p.offsets.data(), ob, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    free_plan(p);
    return hip_fail(e);
  }
  g_plans.push_back(std::move(p));
  *out = &g_plans.back();
  return INTSGD_OK;
}

// What a tiled launch needs: the map, the grid and (multi-block) the device tables.
struct Tiling {
  TileMap tm;
  LaunchShape ls;
  const uint32_t* tile_prefix;
  const uint64_t* offsets_dev;
};

void use_xcd_runs(Tiling* t, uint32_t from_tiles = kXcdRunFromTiles) {
  if (t->tm.num_tiles >= from_tiles) t->tm.xcd_shift = kXcdRunShift;
}

// Dynamic LDS that makes exactly k workgroups fit a CU (0 when k is no cap).
uint32_t lds_reserve_for(uint32_t k) {
  if (k == 0 || k >= 8) return 0;
  return kLdsPerCu / (k + 1) + 1024u;
}

// Automatic tile of the per-worker compress kernel.  Measured on MI355X (one worker,
// d = 108 M): the byte-wide wire wants more coordinates per workgroup (its stores are a
// quarter as wide), randomized rounding more again.
uint32_t compress_tile(const intsgd_desc* desc) {
  const bool random = desc->rounding == INTSGD_ROUND_STOCHASTIC;
  if (desc->wire == INTSGD_WIRE_INT8) return random ? 16384u : 8192u;
  return random ? 8192u : 2048u;
}

// Automatic tiles of the other kernels (an explicit tile_coords in the launch options wins).
// Measured on MI355X at d = 108 M and d = 25.6 M, fraction of the HBM peak:
// the sweeps over the n gradient streams (F3, F1, momentum form) want more coordinates per
// workgroup the fewer streams a thread has to load from: n = 1: 52 % with 2048, 77 % with 4096,
// 81 % with 8192, 80 % with 16384; n = 2: 66 / 83 / 82 %; n = 4: 79 / 81 / 80 %; n = 5: 84 % with
// 4096, 80 % with 8192; n = 6 and 8: 84 and 87 % with 2048, 81 % with 4096.
uint32_t sweep_tile(const intsgd_desc* desc) {
  return desc->n == 1 ? 8192u : desc->n <= 5 ? 4096u : 2048u;
}
// a5-a6, F2 and a7 (two loads and at most one store per coordinate; d = 108 M): 209 / 194 / 201 us,
// 233 / 195 / 200 us and 149 / 128 / 137 us with 2048 / 4096 / 8192.
constexpr uint32_t kDecodeTile = 4096;
// Algorithm 3's sweep has 2n + 2 loads and n + 2 stores per coordinate.  n = 8: 1.96 ms with 1024,
// 2.04 ms with 2048, 2.07 ms with 4096 at d = 108 M (and 0.427 against 0.439 ms at d = 25.6 M);
// n = 4 and n = 16 are 1-5 % faster with 2048; a vector of more than 2^20 tiles of 1024 would
// exceed the launch grid and lose the one-tile-per-workgroup order (d = 1.3 G: 24.9 against 24.3 ms).
uint32_t diana_tile(const intsgd_desc* desc) {
  const bool mid = desc->n >= 6 && desc->n <= 12;
  return (mid && tiles_of(desc->d, 1024u) + desc->num_blocks <= kMaxGrid) ? 1024u : 2048u;
}

intsgd_status make_tiling(const intsgd_desc* desc, void* stream, Tiling* t,
                          uint32_t automatic_tile = 0, bool may_build = true) {
  const Tuning tune = effective_tuning(desc);
  // a kernel may have its own automatic tile; an explicit override still wins
  const uint32_t tile =
      (automatic_tile != 0 && requested_tuning(desc).tile_coords == 0) ? automatic_tile : tune.tile_coords;
  t->tm.d = desc->d;
  t->tm.tile = tile;
  if (desc->num_blocks == 1) {
    t->tm.num_tiles = (uint32_t)tiles_of(desc->d, tile);
    t->tm.table = nullptr;
    t->tile_prefix = nullptr;
    t->offsets_dev = nullptr;
  } else {
    const DevicePlan* plan = nullptr;
    const intsgd_status st = get_plan(desc, tile, &plan, may_build);
    if (st != INTSGD_OK) return st;
    t->tm.num_tiles = plan->num_tiles;
    t->tm.table = plan->table;
    t->tile_prefix = plan->tile_prefix;
    t->offsets_dev = plan->offsets_dev;
  }
  t->tm.xcd_shift = 0;
  t->ls.grid = t->tm.num_tiles < tune.max_workgroups ? t->tm.num_tiles : tune.max_workgroups;
  t->ls.lds_reserve = lds_reserve_for(tune.workgroups_per_cu);
  t->ls.stream = static_cast<hipStream_t>(stream);
  take_taps(desc, &t->ls);
  return INTSGD_OK;
}

void fill_ptrs(WorkerPtrs* w, const void* const* src, uint32_t n) {
  std::memset(w, 0, sizeof(*w));
  for (uint32_t i = 0; i < n; ++i) w->p[i] = src[i];
}

// Ids that tag the clip hint of a launch: non-zero and different from call to call.
uint32_t next_launch_id() {
  static std::atomic<uint32_t> counter{0};
  uint32_t id = ++counter;
  if (id == 0) id = ++counter;
  return id;
}

// The end-of-kernel reduction descriptor.  norm_sq_out / sat_count may be null when the
// kernel does not produce them.
Finish make_finish(const intsgd_desc* desc, const Tiling& t, void* ws, double* norm_sq_out,
                   uint64_t* sat_count, const WorkspaceLayout* layout = nullptr) {
  const WorkspaceLayout w = layout ? *layout : workspace_layout(desc);
  Finish f{};
  f.norm_partial = ws_at<double>(ws, w.norm_off);
  f.norm_mid = ws_at<double>(ws, w.mid_off);
  f.sat_hint = ws_at<uint32_t>(ws, w.hint_off);
  f.launch_id = next_launch_id();
  f.tile_prefix = t.tile_prefix;
  f.num_tiles = t.tm.num_tiles;
  f.B = desc->num_blocks;
  f.norm_sq_out = norm_sq_out;
  f.workgroups = t.ls.grid;
  f.sat_any = ws_at<uint32_t>(ws, w.any_off);
  f.sat_rows = ws_at<uint64_t>(ws, w.rows_off);
  f.n = desc->n;
  f.sat_count = sat_count;
  f.n_workers = desc->n;
  f.d = desc->d;
  f.rule = AlphaRule{nullptr, nullptr, nullptr, 0.0, 0.0, 0.0};
  f.big_partial = ws_at<uint32_t>(ws, w.big_off);
  f.big_mid = ws_at<uint32_t>(ws, w.bigmid_off);
  f.big_out = nullptr;            // set by the calls whose sweep forms the aggregate
  return f;
}

intsgd_status done(hipError_t e) { return e == hipSuccess ? INTSGD_OK : hip_fail(e); }

#define INTSGD_TRY(expr)                        \
  do {                                          \
    const intsgd_status st_ = (expr);           \
    if (st_ != INTSGD_OK) return st_;           \
  } while (0)

}  // namespace
}  // namespace intsgd

using namespace intsgd;

namespace {

// Shared body of intsgd_step_fused and intsgd_step_fused_next_alpha.
intsgd_status validate_momentum(const Momentum* mom) {
  if (mom == nullptr) return INTSGD_OK;
  INTSGD_TRY(validate_vec(mom->m));
  if (!(mom->mu >= 0.0 && mom->mu < 1.0)) return INTSGD_EINVAL;
  if (!(mom->wd >= 0.0) || !std::isfinite(mom->wd)) return INTSGD_EINVAL;
  return INTSGD_OK;
}

// Decides the form of a sweep for this call and, for the two-phase form, its grid.
intsgd_status two_phase_shape(const intsgd_desc* desc, PhasedShape* ps, bool* phased) {
  *phased = false;
  if (!use_two_phase(desc, effective_tuning(desc))) return INTSGD_OK;
  INTSGD_TRY(compute_units(&ps->grid));
  // the caller's workspace holds one slot per 1024 coordinates; one per CU is needed
  *phased = ps->grid <= tiles_of(desc->d, kMinTile);
  return INTSGD_OK;
}

// use_static_scratch: the variant that must not allocate.  Its scratch is the library's
// static device array (workspace arguments ignored), laid out for the tiling this very call
// uses, and a partition's tile table is looked up but never built.
intsgd_status step_fused_impl(const intsgd_desc* desc, const float* const* grads,
                              const float* alpha, double eta, float* x, double* norm_sq_out,
                              uint64_t* sat_count, void* workspace, size_t workspace_bytes,
                              void* hip_stream, double* r, float* alpha_out, double beta,
                              double eps, double eta_next, const Momentum* mom = nullptr,
                              bool use_static_scratch = false) {
  INTSGD_TRY(validate_desc(desc));
  INTSGD_TRY(validate_worker_ptrs((const void* const*)grads, desc->n));
  INTSGD_TRY(validate_vec(x));
  if (alpha == nullptr || norm_sq_out == nullptr || sat_count == nullptr) return INTSGD_EINVAL;
  INTSGD_TRY(validate_rule(beta, eps, eta));
  if (r != nullptr) INTSGD_TRY(validate_rule(beta, eps, eta_next));
  INTSGD_TRY(validate_momentum(mom));
  if (!use_static_scratch) INTSGD_TRY(validate_workspace(desc, workspace, workspace_bytes));
  Tiling t;
  INTSGD_TRY(make_tiling(desc, hip_stream, &t, sweep_tile(desc), /*may_build=*/!use_static_scratch));
  use_xcd_runs(&t, (desc->rounding == INTSGD_ROUND_STOCHASTIC && mom == nullptr)
                       ? kXcdRunFromTilesRandomFused : kXcdRunFromTiles);
  PhasedShape ps{0};
  bool phased = false;
  INTSGD_TRY(two_phase_shape(desc, &ps, &phased));
  WorkspaceLayout layout = workspace_layout(desc);
  if (use_static_scratch) {
    layout = workspace_layout_for(desc, phased ? ps.grid : t.tm.num_tiles);
    if (layout.total > INTSGD_STATIC_SCRATCH_BYTES) return INTSGD_EWORKSPACE;
    const hipError_t e = static_scratch(&workspace);
    if (e != hipSuccess) return hip_fail(e);
  }
  WorkerPtrs g;
  fill_ptrs(&g, (const void* const*)grads, desc->n);
  Finish fin = make_finish(desc, t, workspace, norm_sq_out, sat_count, &layout);
  fin.big_out = desc->largest_sum;
  // Algorithm 1's scaling-factor line pairs alpha_{k+1} with eta_{k+1}
  if (r != nullptr) fin.rule = AlphaRule{r, alpha_out, t.offsets_dev, beta, eps, eta_next};
  if (phased)
    return done(launch_step_fused_phased(ps, t.ls, desc->d, desc->n, round_spec(desc), g, alpha, eta,
                                         x, mom, fin));
  return done(launch_step_fused(t.tm, t.ls, desc->n, round_spec(desc), g, alpha, eta, x, mom, fin));
}

}  // namespace

extern "C" {

size_t intsgd_workspace_bytes(const intsgd_desc* desc) {
  if (validate_desc(desc) != INTSGD_OK) return 0;
  return workspace_layout(desc).total;
}

intsgd_status intsgd_prepare(const intsgd_desc* desc) {
  INTSGD_TRY(validate_desc(desc));
  {   // resolve this device's static scratch array now, so that intsgd_step_fused_static only enqueues
    void* scratch = nullptr;
    uint32_t cus = 0;
    const hipError_t e = static_scratch(&scratch);
    if (e != hipSuccess) return hip_fail(e);
    INTSGD_TRY(compute_units(&cus));
  }
  if (desc->num_blocks == 1) return INTSGD_OK;
  const DevicePlan* plan = nullptr;
  const uint32_t fixed = requested_tuning(desc).tile_coords;
  if (fixed != 0) return get_plan(desc, fixed, &plan);
  // every automatic tile an entry point may pick for this descriptor
  const uint32_t tiles[] = {sweep_tile(desc), compress_tile(desc), kDecodeTile, diana_tile(desc),
                            effective_tuning(desc).tile_coords};
  for (uint32_t tile : tiles) INTSGD_TRY(get_plan(desc, tile, &plan));
  return INTSGD_OK;
}

void intsgd_release(void) {
  std::lock_guard<std::mutex> lock(g_mutex);
  for (DevicePlan& p : g_plans) free_plan(p);
  g_plans.clear();
}

intsgd_status intsgd_compress(const intsgd_desc* desc, const float* const* grads,
                              const float* alpha, void* const* q_out, uint64_t* sat_count,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  INTSGD_TRY(validate_desc(desc));
  INTSGD_TRY(validate_worker_ptrs((const void* const*)grads, desc->n));
  INTSGD_TRY(validate_worker_ptrs((const void* const*)q_out, desc->n));
  if (alpha == nullptr || sat_count == nullptr) return INTSGD_EINVAL;
  INTSGD_TRY(validate_workspace(desc, workspace, workspace_bytes));
  Tiling t;
  INTSGD_TRY(make_tiling(desc, hip_stream, &t, compress_tile(desc)));
  use_xcd_runs(&t);
  WorkerPtrs g;
  WorkerOutPtrs q;
  fill_ptrs(&g, (const void* const*)grads, desc->n);
  std::memset(&q, 0, sizeof(q));
  for (uint32_t i = 0; i < desc->n; ++i) q.p[i] = q_out[i];
  const WorkspaceLayout w = workspace_layout(desc);
  // one read and one write stream per workgroup: a copy-like kernel, which wants every
  // wavefront slot filled (80 % of peak against 62 % under the sweeps' residency cap)
  if (requested_tuning(desc).workgroups_per_cu == 0) t.ls.lds_reserve = 0;
  return done(launch_compress(t.tm, t.ls, desc->n, desc->wire, round_spec(desc), g, alpha, q,
                              ws_at<uint64_t>(workspace, w.rows_off), sat_count));
}

intsgd_status intsgd_int_sum(const intsgd_desc* desc, const void* const* q, int32_t* sum_out,
                             void* hip_stream) {
  INTSGD_TRY(validate_desc(desc));
  INTSGD_TRY(validate_worker_ptrs(q, desc->n));
  INTSGD_TRY(validate_vec(sum_out));
  WorkerPtrs qp;
  fill_ptrs(&qp, q, desc->n);
  // Long vectors take the two-phase form (int8: 16 coordinates per 16-byte load, 51 us against
  // 77 us on 8 x 25.6 M; int32: 0.258 ms against 0.288 ms on 16 x 25.6 M behind intsgd_compress,
  // 0.254 ms against 0.289 ms on its own), unless the tuning asks for the tile form.
  if (desc->d >= kMinPhasedD && effective_tuning(desc).two_phase != 1) {
    PhasedShape ps{0};
    INTSGD_TRY(compute_units(&ps.grid));
    LaunchShape pls{ps.grid, 0, static_cast<hipStream_t>(hip_stream), nullptr, nullptr};
    take_taps(desc, &pls);
    return done(launch_int_sum_phased(ps, pls, desc->d, desc->n, desc->wire, qp, sum_out));
  }
  // one workgroup per 512 quads (at least one, for the d mod 4 coordinates of a tiny vector)
  const uint64_t want = tiles_of((desc->d >> 2) + 1, INTSGD_THREADS_PER_WORKGROUP);
  LaunchShape ls{(uint32_t)want, 0, static_cast<hipStream_t>(hip_stream), nullptr, nullptr};
  take_taps(desc, &ls);
  return done(launch_int_sum(desc->d, ls, desc->n, desc->wire, qp, sum_out));
}

intsgd_status intsgd_decode_update(const intsgd_desc* desc, const int32_t* sum,
                                   const float* alpha, double eta, float* x, float* gtilde_out,
                                   void* hip_stream) {
  INTSGD_TRY(validate_desc(desc));
  INTSGD_TRY(validate_vec(sum));
  INTSGD_TRY(validate_vec(x));
  if (gtilde_out != nullptr) INTSGD_TRY(validate_vec(gtilde_out));
  if (alpha == nullptr) return INTSGD_EINVAL;
  INTSGD_TRY(validate_rule(0.0, 0.0, eta));
  Tiling t;
  INTSGD_TRY(make_tiling(desc, hip_stream, &t, kDecodeTile));
  return done(launch_decode_update(t.tm, t.ls, desc->n, sum, alpha, eta, x, gtilde_out));
}

intsgd_status intsgd_update_norm(const intsgd_desc* desc, const float* x_new, const float* x_old,
                                 double* norm_sq_out, void* workspace, size_t workspace_bytes,
                                 void* hip_stream) {
  INTSGD_TRY(validate_desc(desc));
  INTSGD_TRY(validate_vec(x_new));
  INTSGD_TRY(validate_vec(x_old));
  if (norm_sq_out == nullptr) return INTSGD_EINVAL;
  INTSGD_TRY(validate_workspace(desc, workspace, workspace_bytes));
  Tiling t;
  INTSGD_TRY(make_tiling(desc, hip_stream, &t, kDecodeTile));
  return done(launch_update_norm(t.tm, t.ls, x_new, x_old,
                                 make_finish(desc, t, workspace, norm_sq_out, nullptr)));
}

intsgd_status intsgd_next_alpha(const intsgd_desc* desc, const double* norm_sq, double* r,
                                double beta, double eps, double eta, float* alpha_out,
                                void* hip_stream) {
  INTSGD_TRY(validate_desc(desc));
  if (norm_sq == nullptr || r == nullptr || alpha_out == nullptr) return INTSGD_EINVAL;
  INTSGD_TRY(validate_rule(beta, eps, eta));
  const uint64_t* offsets_dev = nullptr;
  if (desc->num_blocks > 1) {
    const DevicePlan* plan = nullptr;
    INTSGD_TRY(get_plan(desc, effective_tuning(desc).tile_coords, &plan));
    offsets_dev = plan->offsets_dev;
  }
  const AlphaRule rule{r, alpha_out, offsets_dev, beta, eps, eta};
  return done(launch_next_alpha(static_cast<hipStream_t>(hip_stream), norm_sq, rule,
                                desc->num_blocks, desc->n, desc->d));
}

intsgd_status intsgd_next_alpha_host(const intsgd_desc* desc, const double* norm_sq, double* r,
                                     double beta, double eps, double eta, float* alpha_out) {
  INTSGD_TRY(validate_desc(desc));
  if (norm_sq == nullptr || r == nullptr || alpha_out == nullptr) return INTSGD_EINVAL;
  INTSGD_TRY(validate_rule(beta, eps, eta));
  const uint32_t B = desc->num_blocks;
  bool zero_den = false;
  for (uint32_t l = 0; l < B; ++l) {
    const double keep = beta * r[l];
    const double fresh = (1.0 - beta) * norm_sq[l];
    const double rl = keep + fresh;
    r[l] = rl;
    double alpha;
    if (B == 1) {
      const double den = 2.0 * (double)desc->n * rl / (eta * eta) + eps * eps;
      zero_den |= (den == 0.0);
      alpha = std::sqrt((double)desc->d) / std::sqrt(den);
    } else {
      const double dl = (double)(desc->block_offsets[l + 1] - desc->block_offsets[l]);
      const double den = 2.0 * (double)desc->n * rl + eta * eta * (dl / (double)desc->d) * eps * eps;
      zero_den |= (den == 0.0);
      alpha = eta * std::sqrt(dl) / std::sqrt(den);
    }
    alpha_out[l] = (float)alpha;
  }
  return zero_den ? INTSGD_ERANGE : INTSGD_OK;
}

intsgd_status intsgd_compress_sum(const intsgd_desc* desc, const float* const* grads,
                                  const float* alpha, int32_t* sum_out, uint64_t* sat_count,
                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  INTSGD_TRY(validate_desc(desc));
  INTSGD_TRY(validate_worker_ptrs((const void* const*)grads, desc->n));
  INTSGD_TRY(validate_vec(sum_out));
  if (alpha == nullptr || sat_count == nullptr) return INTSGD_EINVAL;
  INTSGD_TRY(validate_workspace(desc, workspace, workspace_bytes));
  Tiling t;
  INTSGD_TRY(make_tiling(desc, hip_stream, &t, sweep_tile(desc)));
  use_xcd_runs(&t);
  WorkerPtrs g;
  fill_ptrs(&g, (const void* const*)grads, desc->n);
  Finish fin = make_finish(desc, t, workspace, nullptr, sat_count);
  fin.big_out = desc->largest_sum;
  PhasedShape ps{0};
  bool phased = false;
  INTSGD_TRY(two_phase_shape(desc, &ps, &phased));
  if (phased)
    return done(launch_compress_sum_phased(ps, t.ls, desc->d, desc->n, round_spec(desc), g, alpha,
                                           sum_out, fin));
  return done(launch_compress_sum(t.tm, t.ls, desc->n, round_spec(desc), g, alpha, sum_out, fin));
}

intsgd_status intsgd_decode_update_norm(const intsgd_desc* desc, const int32_t* sum,
                                        const float* alpha, double eta, float* x,
                                        double* norm_sq_out, void* workspace,
                                        size_t workspace_bytes, void* hip_stream) {
  INTSGD_TRY(validate_desc(desc));
  INTSGD_TRY(validate_vec(sum));
  INTSGD_TRY(validate_vec(x));
  if (alpha == nullptr || norm_sq_out == nullptr) return INTSGD_EINVAL;
  INTSGD_TRY(validate_rule(0.0, 0.0, eta));
  INTSGD_TRY(validate_workspace(desc, workspace, workspace_bytes));
  Tiling t;
  INTSGD_TRY(make_tiling(desc, hip_stream, &t, kDecodeTile));
  return done(launch_decode_update_norm(t.tm, t.ls, desc->n, sum, alpha, eta, x, nullptr,
                                        make_finish(desc, t, workspace, norm_sq_out, nullptr)));
}

intsgd_status intsgd_decode_update_momentum(const intsgd_desc* desc, const int32_t* sum,
                                            const float* alpha, double eta, double mu,
                                            double weight_decay, float* x, float* m,
                                            double* norm_sq_out, void* workspace,
                                            size_t workspace_bytes, void* hip_stream) {
  INTSGD_TRY(validate_desc(desc));
  INTSGD_TRY(validate_vec(sum));
  INTSGD_TRY(validate_vec(x));
  if (alpha == nullptr || norm_sq_out == nullptr) return INTSGD_EINVAL;
  INTSGD_TRY(validate_rule(0.0, 0.0, eta));
  const Momentum mom{m, mu, weight_decay};
  INTSGD_TRY(validate_momentum(&mom));
  INTSGD_TRY(validate_workspace(desc, workspace, workspace_bytes));
  Tiling t;
  INTSGD_TRY(make_tiling(desc, hip_stream, &t, kDecodeTile));
  return done(launch_decode_update_norm(t.tm, t.ls, desc->n, sum, alpha, eta, x, &mom,
                                        make_finish(desc, t, workspace, norm_sq_out, nullptr)));
}

intsgd_status intsgd_step_momentum(const intsgd_desc* desc, const float* const* grads,
                                   float* alpha, double eta, double eta_next, double mu,
                                   double weight_decay, float* x, float* m, double* r, double beta,
                                   double eps, double* norm_sq_out, uint64_t* sat_count,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  const Momentum mom{m, mu, weight_decay};
  return step_fused_impl(desc, grads, alpha, eta, x, norm_sq_out, sat_count, workspace,
                         workspace_bytes, hip_stream, r, alpha, r ? beta : 0.0, r ? eps : 0.0,
                         r ? eta_next : eta, &mom);
}

intsgd_status intsgd_step_fused(const intsgd_desc* desc, const float* const* grads,
                                const float* alpha, double eta, float* x, double* norm_sq_out,
                                uint64_t* sat_count, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
  return step_fused_impl(desc, grads, alpha, eta, x, norm_sq_out, sat_count, workspace,
                         workspace_bytes, hip_stream, nullptr, nullptr, 0.0, 0.0, eta);
}

intsgd_status intsgd_step_fused_next_alpha(const intsgd_desc* desc, const float* const* grads,
                                           float* alpha, double eta, double eta_next, float* x,
                                           double* r, double beta, double eps, double* norm_sq_out,
                                           uint64_t* sat_count, void* workspace,
                                           size_t workspace_bytes, void* hip_stream) {
  if (r == nullptr) return INTSGD_EINVAL;
  return step_fused_impl(desc, grads, alpha, eta, x, norm_sq_out, sat_count, workspace,
                         workspace_bytes, hip_stream, r, alpha, beta, eps, eta_next);
}

intsgd_status intsgd_step_fused_static(const intsgd_desc* desc, const float* const* grads,
                                       float* alpha, double eta, double eta_next, float* x,
                                       double* r, double beta, double eps, double* norm_sq_out,
                                       uint64_t* sat_count, void* hip_stream) {
  if (r == nullptr) return INTSGD_EINVAL;
  return step_fused_impl(desc, grads, alpha, eta, x, norm_sq_out, sat_count, nullptr, 0, hip_stream,
                         r, alpha, beta, eps, eta_next, nullptr, /*use_static_scratch=*/true);
}

intsgd_status intsgd_diana_step(const intsgd_desc* desc, const float* const* grads,
                                float* const* h_local, float* alpha, double eta, double eta_next,
                                float* x, float* h, double* r, double beta, double eps,
                                double* norm_sq_out, uint64_t* sat_count, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  INTSGD_TRY(validate_desc(desc));
  INTSGD_TRY(validate_worker_ptrs((const void* const*)grads, desc->n));
  INTSGD_TRY(validate_worker_ptrs((const void* const*)h_local, desc->n));
  INTSGD_TRY(validate_vec(x));
  INTSGD_TRY(validate_vec(h));
  if (alpha == nullptr || norm_sq_out == nullptr || sat_count == nullptr) return INTSGD_EINVAL;
  INTSGD_TRY(validate_rule(r ? beta : 0.0, r ? eps : 0.0, eta));
  if (r != nullptr) INTSGD_TRY(validate_rule(beta, eps, eta_next));
  INTSGD_TRY(validate_workspace(desc, workspace, workspace_bytes));
  Tiling t;
  INTSGD_TRY(make_tiling(desc, hip_stream, &t, diana_tile(desc)));
  use_xcd_runs(&t);
  WorkerPtrs g;
  WorkerOutPtrs hl;
  fill_ptrs(&g, (const void* const*)grads, desc->n);
  std::memset(&hl, 0, sizeof(hl));
  for (uint32_t i = 0; i < desc->n; ++i) hl.p[i] = h_local[i];
  Finish fin = make_finish(desc, t, workspace, norm_sq_out, sat_count);
  fin.big_out = desc->largest_sum;
  if (r != nullptr) fin.rule = AlphaRule{r, alpha, t.offsets_dev, beta, eps, eta_next};
  return done(launch_diana_step(t.tm, t.ls, desc->n, round_spec(desc), g, hl, alpha, eta, x, h, fin));
}

intsgd_status intsgd_heuristic_alpha(const intsgd_desc* desc, const float* const* grads,
                                     uint32_t nb, float* alpha_out, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
  INTSGD_TRY(validate_desc(desc));
  INTSGD_TRY(validate_worker_ptrs((const void* const*)grads, desc->n));
  if (alpha_out == nullptr) return INTSGD_EINVAL;
  if (nb < 1 || nb > 31) return INTSGD_ERANGE;
  INTSGD_TRY(validate_workspace(desc, workspace, workspace_bytes));
  Tiling t;
  INTSGD_TRY(make_tiling(desc, hip_stream, &t));
  WorkerPtrs g;
  fill_ptrs(&g, (const void* const*)grads, desc->n);
  const WorkspaceLayout w = workspace_layout(desc);
  return done(launch_heuristic_alpha(t.tm, t.ls, desc->n, nb, g, ws_at<uint32_t>(workspace, w.norm_off),
                                     t.tile_prefix, desc->num_blocks, alpha_out));
}

int intsgd_fused_step_form(const intsgd_desc* desc) {
  if (validate_desc(desc) != INTSGD_OK) return 0;
  return use_two_phase(desc, effective_tuning(desc)) ? 2 : 1;
}

const char* intsgd_status_string(int status) {
  switch (status) {
    case INTSGD_OK: return "ok";
    case INTSGD_EINVAL: return "invalid argument";
    case INTSGD_EALIGN: return "vector pointer not 16-byte aligned";
    case INTSGD_ERANGE: return "value out of range";
    case INTSGD_EHIP: return "HIP runtime error";
    case INTSGD_EWORKSPACE: return "workspace missing, misaligned or too small";
    case INTSGD_ENOPLAN: return "partition not prepared (intsgd_prepare) and this call must not allocate";
  }
  return "unknown status";
}

const char* intsgd_last_hip_error(void) { return t_hip_error.c_str(); }

}  // extern "C"
