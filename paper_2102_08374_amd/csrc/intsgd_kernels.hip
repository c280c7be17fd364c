// HIP kernels of the IntSGD step for gfx950 (CDNA4, 64-wide wavefronts).
//
// The whole path is a streaming scan (no reuse, no dense contraction), so the
// design goal is HBM bandwidth:
//   * every lane moves 16 bytes per stream per access (buffer_load/store_dwordx4)
//     through a wave-uniform buffer descriptor + 32-bit lane offset; the descriptor
//     covers exactly the tile, so a stray lane offset cannot leave it;
//   * gradient streams are read non-temporally, up to 8 independent loads in flight
//     per lane; x is written through (sc1) so that no dirty lines pile up in L2;
//   * the integer aggregate stays in registers in the fused forms;
//   * two forms of the fused sweep.  Tile sweep (any partition, both rounding modes): a
//     workgroup is 512 threads and handles ONE tile of 2048 or 4096 coordinates, and
//     residency is capped (by an LDS reservation) at two or four workgroups per CU:
//     with a write stream mixed into the reads, fewer, larger requests in flight measured
//     faster than full occupancy.  Two-phase sweep (one block): one persistent workgroup
//     of 1024 threads per CU alternates between reading the gradient streams, with the
//     sums of 12 quads per thread kept in registers, and updating x for the same quads,
//     so that the chip as a whole alternates between a read-only stream and a short
//     read-modify-write burst;
//   * the sweep writes one norm partial per tile (or workgroup) and, only where something
//     clipped, a row of clip counts per workgroup; a small kernel right behind it on the
//     stream sums them in a fixed order and applies the alpha rule.  (Electing the
//     sweep's last workgroup through a ticket instead was measured 3x slower with one
//     workgroup per tile, and brings nothing with one workgroup per CU: consecutive
//     launches on a stream already hide the small kernel's dispatch.)
//
// Work is cut into tiles that never straddle a block of Algorithm 2, so alpha is
// wave-uniform inside a tile.  A tile whose ends are not multiples of four
// coordinates handles its <= 3 head and <= 3 tail coordinates one by one;
// everything in between moves as aligned quads.

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <mutex>
#include <vector>

#include "intsgd_internal.h"

// Scratch memory of intsgd_step_fused_static, the entry point for callers that cannot
// allocate: norm partials, clip flags and clip-count rows of one call.  Every GPU that loads
// the library holds its own copy of this array, at its own address, until the process ends.
// In host code the name below is only a stand-in for the symbol: kernels get the address
// that hipGetSymbolAddress returns for the current device (static_scratch()).
static __device__ __align__(256) unsigned char scratch[INTSGD_STATIC_SCRATCH_BYTES];

namespace intsgd {

hipError_t static_scratch(void** ptr) {
  static std::mutex m;
  static std::vector<void*> per_device;
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(m);
  if ((size_t)device >= per_device.size()) per_device.resize((size_t)device + 1, nullptr);
  if (per_device[device] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    per_device[device] = p;
  }
  *ptr = per_device[device];
  return hipSuccess;
}

namespace {

constexpr uint32_t kThreads = INTSGD_THREADS_PER_WORKGROUP;
constexpr uint32_t kPhasedThreads = 1024;     // one workgroup per CU in the two-phase sweep
// quads whose integer sums a thread keeps in registers (fewer with Philox's temporaries)
constexpr uint32_t phased_quads(int rounding) { return rounding == INTSGD_ROUND_STOCHASTIC ? 8u : 12u; }
constexpr uint32_t kMaxWaves = kPhasedThreads / 64;

// Native 16-byte vectors (one dwordx4 access each).
typedef float vf4 __attribute__((ext_vector_type(4)));
typedef int32_t vi4 __attribute__((ext_vector_type(4)));
typedef uint32_t vu4 __attribute__((ext_vector_type(4)));

// Cache-policy bits of buffer instructions on gfx950 (the aux operand).
constexpr int kPlain = 0;
constexpr int kNonTemporal = 2;    // nt: streaming data, not reused
constexpr int kWriteThrough = 16;  // sc1: store goes through L2 to memory
constexpr int kStreamOut = 18;     // nt + sc1: written through and not kept (vectors beyond the last-level cache)

#ifndef INTSGD_GRAD_LOAD_POLICY
#define INTSGD_GRAD_LOAD_POLICY kNonTemporal
#endif
#ifndef INTSGD_X_LOAD_POLICY
#define INTSGD_X_LOAD_POLICY kPlain
#endif
#ifndef INTSGD_X_STORE_POLICY
#define INTSGD_X_STORE_POLICY kWriteThrough
#endif
// 0 = randomized rounding clamps and tests every coordinate (A/B builds only)
#ifndef INTSGD_RANDOM_FAST_PATH
#define INTSGD_RANDOM_FAST_PATH 1
#endif

// ------------------------------------------------------------------ buffer access
// Raw buffer descriptor over [base, base+bytes): dword 3 = 0x00020000 selects the
// 32-bit raw format on gfx90a/gfx94x/gfx950.  Out-of-range lanes read 0 / are dropped.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_stream(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
template <int POLICY>
__device__ __forceinline__ vu4 load128(__amdgpu_buffer_rsrc_t s, uint32_t byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(s, (int)byte_off, 0, POLICY);
}
template <int POLICY>
__device__ __forceinline__ void store128(__amdgpu_buffer_rsrc_t s, uint32_t byte_off, vu4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, s, (int)byte_off, 0, POLICY);
}
template <int POLICY>
__device__ __forceinline__ void store32(__amdgpu_buffer_rsrc_t s, uint32_t byte_off, uint32_t v) {
  __builtin_amdgcn_raw_buffer_store_b32(v, s, (int)byte_off, 0, POLICY);
}
__device__ __forceinline__ vf4 as_f(vu4 v) { return __builtin_bit_cast(vf4, v); }
__device__ __forceinline__ vi4 as_i(vu4 v) { return __builtin_bit_cast(vi4, v); }
__device__ __forceinline__ vu4 as_u(vf4 v) { return __builtin_bit_cast(vu4, v); }
__device__ __forceinline__ vu4 as_u(vi4 v) { return __builtin_bit_cast(vu4, v); }

// ------------------------------------------------------------------ Philox4x32-10
// Counter-based generator of Salmon et al. (SC'11), written from its description:
// ten rounds of two 32x32->64 multiplies, a word permutation and key injection,
// with the key bumped by Weyl constants between rounds.  On gfx950 the 32-bit
// multiplies issue at full rate, so the two three-way xors of a round are half of its
// cost as plain xors; v_bitop3_b32 (truth table 0x96 = a ^ b ^ c) does each in one.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

struct PhiloxState {
  uint32_t c0, c1, c2, c3, k0, k1;
};

__device__ __forceinline__ void philox_bump_key(PhiloxState& s) {
  s.k0 += 0x9E3779B9u;
  s.k1 += 0xBB67AE85u;
}

// PRECONDITION: c2, c3 and the key are wave-uniform (worker, step and seed at every call
// site); (c0, c1) is per lane.  In the first round two operands of each three-way xor are
// then uniform, in the second round two operands of one of them; the uniform pair is
// combined on the scalar unit (readfirstlane pins it there: the compiler otherwise
// reassociates the xors back onto the vector unit), leaving one vector xor each.
__device__ __forceinline__ vu4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                             uint32_t k0, uint32_t k1) {
  PhiloxState s{c0, c1, c2, c3, k0, k1};
  {
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)s.c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)s.c2;
    const uint32_t n0 = s.c1 ^ __builtin_amdgcn_readfirstlane((uint32_t)(p1 >> 32) ^ s.k0);
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ __builtin_amdgcn_readfirstlane(s.c3 ^ s.k1);
    s.c1 = (uint32_t)p1;
    s.c3 = (uint32_t)p0;
    s.c0 = n0;
    s.c2 = n2;
    philox_bump_key(s);
  }
  {
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)s.c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)s.c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ __builtin_amdgcn_readfirstlane(s.c1 ^ s.k0);
    const uint32_t n2 = xor3((uint32_t)(p0 >> 32), s.c3, s.k1);
    s.c1 = (uint32_t)p1;
    s.c3 = (uint32_t)p0;
    s.c0 = n0;
    s.c2 = n2;
    philox_bump_key(s);
  }
#pragma unroll
  for (int round = 2; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)s.c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)s.c2;
    const uint32_t n0 = xor3((uint32_t)(p1 >> 32), s.c1, s.k0);
    const uint32_t n2 = xor3((uint32_t)(p0 >> 32), s.c3, s.k1);
    s.c1 = (uint32_t)p1;
    s.c3 = (uint32_t)p0;
    s.c0 = n0;
    s.c2 = n2;
    philox_bump_key(s);
  }
  return vu4{s.c0, s.c1, s.c2, s.c3};
}

__device__ __forceinline__ uint32_t pick_word(const vu4& w, uint32_t c) {
  return c == 0 ? w.x : (c == 1 ? w.y : (c == 2 ? w.z : w.w));
}

// ------------------------------------------------------------------ rounding + clip
// v_cvt_i32_f32 saturates out-of-range inputs and maps NaN to 0, which is the clip
// contract's behaviour; a C++ cast would be undefined there.
__device__ __forceinline__ int32_t cvt_i32_saturating(float r) {
  int32_t q;
  asm("v_cvt_i32_f32_e32 %0, %1" : "=v"(q) : "v"(r));
  return q;
}

// Clamp to [-L, L] (L >= 1, wave-uniform) as one median-of-three; the compiler cannot
// form it from min/max because it cannot prove -L <= L.  Only one operand may be an
// SGPR on this ISA, hence L in a VGPR.
__device__ __forceinline__ int32_t clamp_sym(int32_t q, int32_t L) {
  // The copy of L is an asm of its own so that it is made once and kept: a plain "v"(L)
  // operand is re-created from the SGPR before every use (one v_mov per coordinate).
  int32_t lv, r;
  asm("v_mov_b32 %0, %1" : "=v"(lv) : "s"(L));
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(q), "s"(-L), "v"(lv));
  return r;
}

// Clip events are kept as wavefront lane masks: the compares below write an SGPR pair
// directly, masks combine and are counted on the scalar unit, and no vector
// instruction is spent on turning a per-lane flag back into a mask.
typedef unsigned long long LaneMask;
constexpr int kFcmpNotLess = 11;   // unordered or >=
constexpr int kIcmpNotEqual = 33;

__device__ __forceinline__ bool lane_in(LaneMask m) {
  return ((m >> (threadIdx.x & 63u)) & 1ull) != 0ull;
}

__device__ __forceinline__ uint32_t count_lanes(LaneMask m0, LaneMask m1, LaneMask m2, LaneMask m3) {
  if ((m0 | m1 | m2 | m3) == 0ull) return 0u;
  return (uint32_t)(__builtin_popcountll(m0) + __builtin_popcountll(m1) +
                    __builtin_popcountll(m2) + __builtin_popcountll(m3));
}

// Section 5.1 deterministic rounding (nearest, ties to even) of t = alpha*g, clipped
// to [-L, L].  `sat` = lanes whose rounded value did not fit (or was not finite).
__device__ __forceinline__ int32_t round_nearest_clip(float t, const RoundSpec& rs, LaneMask& sat) {
  const float r = __builtin_rintf(t);
  sat = __builtin_amdgcn_fcmpf(__builtin_fabsf(r), rs.sat_threshold, kFcmpNotLess);
  return clamp_sym(cvt_i32_saturating(r), rs.clip);
}

// Section 2 randomized rounding Int(t): floor(t)+1 with probability t-floor(t).  The
// draw u = (word>>8) 2^-24 rounds up iff u < p, evaluated as (word>>8) < p 2^24 (both
// sides exact in fp32).
__device__ __forceinline__ int32_t round_random_clip(float t, uint32_t word, const RoundSpec& rs,
                                                     LaneMask& sat) {
  const float f = __builtin_floorf(t);
  const float p = t - f;
  const bool up = (float)(word >> 8) < p * 16777216.0f;
  const int32_t q = cvt_i32_saturating(f) + (up ? 1 : 0);   // up is false whenever |f| >= 2^24
  const int32_t qc = clamp_sym(q, rs.clip);
  sat = __builtin_amdgcn_uicmp((uint32_t)qc, (uint32_t)q, kIcmpNotEqual) |
        __builtin_amdgcn_fcmpf(__builtin_fabsf(f), 2147483648.0f, kFcmpNotLess);
  return qc;
}

// The same randomized rounding for values that are known not to clip: floor(t) + [u < p] is
// ADDED to the running sum S (the compare's carry rides on the add), with no clamp and no
// clip test.  Valid only while |t| < L (then the result lies in [-L, L]); the caller tracks
// the range of its t's with a RangeWatch and redoes the quad with round_random_clip if
// any of them might clip or is not finite.
__device__ __forceinline__ void round_random_add(float t, uint32_t word, int32_t& S) {
  const float f = __builtin_floorf(t);
  const float p = t - f;
  const float scaled_p = p * 16777216.0f;
  const float u = (float)(word >> 8);
  const int32_t q = cvt_i32_saturating(f);
  // S += q + [u < p 2^24] as compare + add-with-carry (the compiler makes a select and a
  // three-way add of it, one instruction more per coordinate)
  asm("v_cmp_gt_f32_e32 vcc, %2, %3\n\tv_addc_co_u32_e32 %0, vcc, %0, %1, vcc"
      : "+v"(S)
      : "v"(q), "v"(scaled_p), "v"(u)
      : "vcc");
}

// Largest |t| seen, kept as two integer maxima of the raw bit patterns: as signed integers
// the non-negative floats (and +NaN) order like their values and beat every negative one;
// as unsigned integers the negative floats (and -NaN) order by magnitude and beat every
// non-negative one.  Two three-way maxima per four values, and NaN / Inf cannot hide.
struct RangeWatch {
  int32_t pos;      // max over raw bits as signed
  uint32_t neg;     // max over raw bits as unsigned
};
__device__ __forceinline__ RangeWatch range_watch_init() { return RangeWatch{INT32_MIN, 0u}; }
__device__ __forceinline__ void watch(RangeWatch& rw, const vf4& t) {
  const vi4 b = __builtin_bit_cast(vi4, t);
  rw.pos = max(max(rw.pos, b.x), b.y);
  rw.pos = max(max(rw.pos, b.z), b.w);
  rw.neg = max(max(rw.neg, (uint32_t)b.x), (uint32_t)b.y);
  rw.neg = max(max(rw.neg, (uint32_t)b.z), (uint32_t)b.w);
}
// Lanes whose quad must be redone exactly: some |t| >= the largest fp32 <= L, or not finite.
constexpr int kIcmpUnsignedGe = 35;
constexpr int kIcmpSignedGe = 39;
__device__ __forceinline__ LaneMask out_of_fast_range(const RangeWatch& rw, const RoundSpec& rs) {
  return __builtin_amdgcn_sicmp(rw.pos, (int32_t)rs.fast_limit_bits, kIcmpSignedGe) |
         __builtin_amdgcn_uicmp(rw.neg, rs.fast_limit_bits | 0x80000000u, kIcmpUnsignedGe);
}

template <int ROUND>
__device__ __forceinline__ int32_t round_clip(float t, uint32_t word, const RoundSpec& rs,
                                              LaneMask& sat) {
  if (ROUND == INTSGD_ROUND_STOCHASTIC) return round_random_clip(t, word, rs, sat);
  return round_nearest_clip(t, rs, sat);
}

// ------------------------------------------------------------------ reductions
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  int lo = __double2loint(v);
  int hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xF, 0xF, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xF, 0xF, false);
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double read_lane(double v, int lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
  return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes of a wavefront; every lane must be active.  Four DPP steps
// (quad swaps, half-row mirror, row mirror) leave each 16-lane row holding its row
// sum; the four row sums are then read through SGPRs and added in a fixed order.
__device__ __forceinline__ double wave_sum(double v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);   // row_half_mirror
  v += dpp_move<0x140>(v);   // row_mirror
  return (read_lane(v, 0) + read_lane(v, 16)) + (read_lane(v, 32) + read_lane(v, 48));
}

// LDS shared by the reductions of one kernel.
struct ReduceLds {
  double red[2][kMaxWaves];         // double-buffered wave sums
  unsigned long long sat[INTSGD_MAX_WORKERS];
  uint32_t big[2][kMaxWaves];       // double-buffered wave maxima
};

// Sum over the workgroup, a two-level tree: DPP / lane reads within each wavefront, the wave
// sums through LDS, and the same wavefront tree once more over them in the first wavefront
// (fixed order).  The result is valid in thread 0 only.  `slot` must alternate between
// consecutive calls (double-buffered LDS, one barrier per call).
__device__ __forceinline__ double block_sum(double v, ReduceLds& lds, uint32_t slot) {
  const double w = wave_sum(v);
  if ((threadIdx.x & 63u) == 0) lds.red[slot][threadIdx.x >> 6] = w;
  __syncthreads();
  double total = 0.0;
  if (threadIdx.x < 64u) {          // the whole first wavefront: wave_sum needs all 64 lanes
    const uint32_t waves = blockDim.x >> 6;
    total = wave_sum(threadIdx.x < waves ? lds.red[slot][threadIdx.x] : 0.0);
  }
  return total;
}

// Largest and smallest aggregate a thread has seen: the largest |S_j| is max(hi, -lo).
// Kept as two signed extremes so that a quad costs four three-input min / max instructions.
struct Extremes {
  int32_t hi, lo;
};
__device__ __forceinline__ Extremes extremes_init() { return Extremes{0, 0}; }
__device__ __forceinline__ void note(Extremes& e, int32_t S) {
  e.hi = max(e.hi, S);
  e.lo = min(e.lo, S);
}
__device__ __forceinline__ void note(Extremes& e, const vi4& S) {
  e.hi = max(max(e.hi, S.x), S.y);
  e.hi = max(max(e.hi, S.z), S.w);
  e.lo = min(min(e.lo, S.x), S.y);
  e.lo = min(min(e.lo, S.z), S.w);
}
__device__ __forceinline__ uint32_t magnitude(const Extremes& e) {
  const uint32_t neg = 0u - (uint32_t)e.lo;       // |lo| without overflow at INT32_MIN
  return max((uint32_t)e.hi, neg);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}

// Maximum over the workgroup (same tree as block_sum; exact in any order).  Valid in thread 0;
// `slot` alternates between consecutive calls.
__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
  v = max(v, dpp_move_u32<0xB1>(v));
  v = max(v, dpp_move_u32<0x4E>(v));
  v = max(v, dpp_move_u32<0x141>(v));
  v = max(v, dpp_move_u32<0x140>(v));
  return max(max((uint32_t)__builtin_amdgcn_readlane((int)v, 0), (uint32_t)__builtin_amdgcn_readlane((int)v, 16)),
             max((uint32_t)__builtin_amdgcn_readlane((int)v, 32), (uint32_t)__builtin_amdgcn_readlane((int)v, 48)));
}
__device__ __forceinline__ uint32_t block_max(uint32_t v, ReduceLds& lds, uint32_t slot) {
  const uint32_t w = wave_max(v);
  if ((threadIdx.x & 63u) == 0) lds.big[slot][threadIdx.x >> 6] = w;
  __syncthreads();
  uint32_t total = 0u;
  if (threadIdx.x < 64u) {
    const uint32_t waves = blockDim.x >> 6;
    total = wave_max(threadIdx.x < waves ? lds.big[slot][threadIdx.x] : 0u);
  }
  return total;
}

// block_sum and block_max behind one barrier (valid in thread 0).
__device__ __forceinline__ void block_sum_and_max(double v, uint32_t m, ReduceLds& lds, uint32_t slot,
                                                  double& total, uint32_t& best) {
  const double w = wave_sum(v);
  const uint32_t wm = wave_max(m);
  if ((threadIdx.x & 63u) == 0) {
    lds.red[slot][threadIdx.x >> 6] = w;
    lds.big[slot][threadIdx.x >> 6] = wm;
  }
  __syncthreads();
  total = 0.0;
  best = 0u;
  if (threadIdx.x < 64u) {
    const uint32_t waves = blockDim.x >> 6;
    total = wave_sum(threadIdx.x < waves ? lds.red[slot][threadIdx.x] : 0.0);
    best = wave_max(threadIdx.x < waves ? lds.big[slot][threadIdx.x] : 0u);
  }
}

// ------------------------------------------------------------------ tiles
struct Tile {
  uint64_t start;
  uint32_t len;
  uint32_t blk;
};

__device__ __forceinline__ Tile locate(const TileMap& tm, uint32_t t) {
  Tile tl;
  if (tm.table != nullptr) {
    const TileEntry e = tm.table[t];
    tl.start = e.start;
    tl.len = e.len;
    tl.blk = e.blk;
  } else {
    tl.start = (uint64_t)t * tm.tile;
    const uint64_t rest = tm.d - tl.start;
    tl.len = rest < tm.tile ? (uint32_t)rest : tm.tile;
    tl.blk = 0;
  }
  return tl;
}

// Runs `op` over this workgroup's tiles (grid-stride).  Op provides
//   begin_tile(blk), scalar(j), begin_body(first_quad, quads), quad(lane_quad),
//   end_tile(t, iter).
template <class Op>
__device__ __forceinline__ void drive_tiles(const TileMap& tm, Op& op) {
  const uint32_t tid = threadIdx.x;
  uint32_t iter = 0;
  uint32_t first = blockIdx.x;
  if (tm.xcd_shift != 0u && gridDim.x == tm.num_tiles) {
    // One tile per workgroup, and consecutive workgroups go to the 8 XCDs in turn.  Within every
    // group of 8 << xcd_shift tiles, give each XCD a run of 1 << xcd_shift consecutive tiles
    // instead of every eighth one (a permutation of the group; an incomplete last group keeps
    // the plain order).  Done before the loop so that nothing of it stays live inside.
    const uint32_t gs = 3u + tm.xcd_shift;
    const uint32_t g = first >> gs, r = first & ((1u << gs) - 1u);
    if (((g + 1u) << gs) <= tm.num_tiles) first = (g << gs) + ((r & 7u) << tm.xcd_shift) + (r >> 3);
  }
  for (uint32_t t = first; t < tm.num_tiles; t += gridDim.x, ++iter) {
    const Tile tl = locate(tm, t);
    const uint64_t s = tl.start, e = tl.start + tl.len;
    uint64_t a = (s + 3) & ~(uint64_t)3;
    if (a > e) a = e;
    uint64_t b = e & ~(uint64_t)3;
    if (b < a) b = a;
    op.begin_tile(tl.blk);
    if (s + tid < a) op.scalar(s + tid);
    const uint32_t nq = (uint32_t)((b - a) >> 2);
    op.begin_body(a >> 2, nq);
    for (uint32_t ql = tid; ql < nq; ql += kThreads) op.quad(ql);
    if (b + tid < e) op.scalar(b + tid);
    op.end_tile(t, iter);
  }
}

// ------------------------------------------------------------------ a1-a4 on one quad
// Scales, rounds, clips and accumulates workers [i0, i0+W) for lane quad `ql` of the
// tile body that starts at quad q0 and holds nq quads.  Clip events are rare, and a
// branch per worker in the streaming loop keeps the compiler from moving the next
// group's loads above this group's arithmetic.  So the sweep runs with COUNT = false:
// it only ORs the clip masks into `any` (scalar unit, no branch); a wavefront whose
// `any` is non-zero afterwards goes over its quads once more with COUNT = true, which
// adds the per-worker counts to LDS (the integers of that second pass are discarded).
template <int ROUND, int W, bool COUNT>
__device__ __forceinline__ void accumulate_workers(const WorkerPtrs& grads, uint32_t i0,
                                                   uint64_t q0, uint32_t nq, uint32_t ql,
                                                   float alpha, const RoundSpec& rs, vi4& S,
                                                   unsigned long long* lds_sat, LaneMask& any) {
  vf4 g[W];
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const __amdgpu_buffer_rsrc_t src = make_stream((const vf4*)grads.p[i0 + w] + q0, nq * 16u);
    g[w] = as_f(load128<INTSGD_GRAD_LOAD_POLICY>(src, ql * 16u));
  }
  const uint64_t quad = q0 + ql;
#pragma unroll
  for (int w = 0; w < W; ++w) {
    vu4 rw = vu4{0u, 0u, 0u, 0u};
    if (ROUND == INTSGD_ROUND_STOCHASTIC)
      rw = philox4x32_10((uint32_t)quad, (uint32_t)(quad >> 32), i0 + w, rs.step, rs.key0, rs.key1);
    LaneMask s0, s1, s2, s3;
    S.x += round_clip<ROUND>(alpha * g[w].x, rw.x, rs, s0);
    S.y += round_clip<ROUND>(alpha * g[w].y, rw.y, rs, s1);
    S.z += round_clip<ROUND>(alpha * g[w].z, rw.z, rs, s2);
    S.w += round_clip<ROUND>(alpha * g[w].w, rw.w, rs, s3);
    if (COUNT) {
      const uint32_t cnt = count_lanes(s0, s1, s2, s3);
      if (cnt != 0 && (threadIdx.x & 63u) == 0) atomicAdd(&lds_sat[i0 + w], (unsigned long long)cnt);
    } else {
      any |= (s0 | s1) | (s2 | s3);
    }
  }
}

// Randomized rounding of workers [i0, i0+W) for one lane quad without clamp or clip test
// (round_random_add); `rw` collects the range of the scaled values.
template <int W>
__device__ __forceinline__ void accumulate_workers_fast(const WorkerPtrs& grads, uint32_t i0,
                                                        uint64_t q0, uint32_t nq, uint32_t ql,
                                                        float alpha, const RoundSpec& rs, vi4& S,
                                                        RangeWatch& rw) {
  vf4 g[W];
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const __amdgpu_buffer_rsrc_t src = make_stream((const vf4*)grads.p[i0 + w] + q0, nq * 16u);
    g[w] = as_f(load128<INTSGD_GRAD_LOAD_POLICY>(src, ql * 16u));
  }
  const uint64_t quad = q0 + ql;
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const vu4 word = philox4x32_10((uint32_t)quad, (uint32_t)(quad >> 32), i0 + w, rs.step, rs.key0, rs.key1);
    const vf4 t = vf4{alpha * g[w].x, alpha * g[w].y, alpha * g[w].z, alpha * g[w].w};
    int32_t s0 = S.x, s1 = S.y, s2 = S.z, s3 = S.w;
    round_random_add(t.x, word.x, s0);
    round_random_add(t.y, word.y, s1);
    round_random_add(t.z, word.z, s2);
    round_random_add(t.w, word.w, s3);
    S = vi4{s0, s1, s2, s3};
    watch(rw, t);
    // one worker after the other: left to itself the scheduler interleaves several workers'
    // Philox chains, which costs 25 more VGPRs (and two resident wavefronts per SIMD)
    __builtin_amdgcn_sched_barrier(0);
  }
}

// The n workers of one lane quad by the fast path; `redo` = lanes whose result is not valid
// (something may clip or is not finite): the caller then runs aggregate_quad<.., true>.
__device__ __forceinline__ vi4 aggregate_quad_fast(const WorkerPtrs& grads, uint32_t n, uint64_t q0,
                                                   uint32_t nq, uint32_t ql, float alpha,
                                                   const RoundSpec& rs, LaneMask& redo) {
  vi4 S = vi4{0, 0, 0, 0};
  RangeWatch rw = range_watch_init();
  uint32_t i = 0;
  for (; i + 8 <= n; i += 8) accumulate_workers_fast<8>(grads, i, q0, nq, ql, alpha, rs, S, rw);
  if (n - i >= 4) {
    accumulate_workers_fast<4>(grads, i, q0, nq, ql, alpha, rs, S, rw);
    i += 4;
  }
  if (n - i >= 2) {
    accumulate_workers_fast<2>(grads, i, q0, nq, ql, alpha, rs, S, rw);
    i += 2;
  }
  if (n - i >= 1) accumulate_workers_fast<1>(grads, i, q0, nq, ql, alpha, rs, S, rw);
  redo = out_of_fast_range(rw, rs);
  return S;
}

template <int ROUND, bool COUNT>
__device__ __forceinline__ vi4 aggregate_quad(const WorkerPtrs& grads, uint32_t n, uint64_t q0,
                                              uint32_t nq, uint32_t ql, float alpha,
                                              const RoundSpec& rs, unsigned long long* lds_sat,
                                              LaneMask& any) {
  vi4 S = vi4{0, 0, 0, 0};
  if (!COUNT && ROUND == INTSGD_ROUND_NEAREST_EVEN && n == 16u) {
    // straight-line code for the common n = 16: the second group's loads can be issued
    // while the first group is being rounded
    accumulate_workers<ROUND, 8, COUNT>(grads, 0, q0, nq, ql, alpha, rs, S, lds_sat, any);
    accumulate_workers<ROUND, 8, COUNT>(grads, 8, q0, nq, ql, alpha, rs, S, lds_sat, any);
    return S;
  }
  uint32_t i = 0;
  for (; i + 8 <= n; i += 8)
    accumulate_workers<ROUND, 8, COUNT>(grads, i, q0, nq, ql, alpha, rs, S, lds_sat, any);
  if (n - i >= 4) {
    accumulate_workers<ROUND, 4, COUNT>(grads, i, q0, nq, ql, alpha, rs, S, lds_sat, any);
    i += 4;
  }
  if (n - i >= 2) {
    accumulate_workers<ROUND, 2, COUNT>(grads, i, q0, nq, ql, alpha, rs, S, lds_sat, any);
    i += 2;
  }
  if (n - i >= 1) accumulate_workers<ROUND, 1, COUNT>(grads, i, q0, nq, ql, alpha, rs, S, lds_sat, any);
  return S;
}

// One coordinate of one worker (head / tail of an unaligned tile).
template <int ROUND>
__device__ __forceinline__ int32_t compress_scalar(const void* g, uint64_t j, uint32_t worker,
                                                   float alpha, const RoundSpec& rs, LaneMask& sat) {
  const float gv = ((const float*)g)[j];
  uint32_t word = 0;
  if (ROUND == INTSGD_ROUND_STOCHASTIC) {
    const uint64_t quad = j >> 2;
    const vu4 rw = philox4x32_10((uint32_t)quad, (uint32_t)(quad >> 32), worker, rs.step,
                                 rs.key0, rs.key1);
    word = pick_word(rw, (uint32_t)(j & 3));
  }
  return round_clip<ROUND>(alpha * gv, word, rs, sat);
}

template <int ROUND>
__device__ __forceinline__ int32_t aggregate_scalar(const WorkerPtrs& grads, uint32_t n, uint64_t j,
                                                    float alpha, const RoundSpec& rs,
                                                    unsigned long long* lds_sat) {
  int32_t S = 0;
  for (uint32_t i = 0; i < n; ++i) {
    LaneMask sat;
    S += compress_scalar<ROUND>(grads.p[i], j, i, alpha, rs, sat);
    if (lane_in(sat)) atomicAdd(&lds_sat[i], 1ull);
  }
  return S;
}

// ------------------------------------------------------------------ a5-a7 on one coordinate
// fp64: x_new = fl32(x - c S); returns x_new and adds (x_new - x)^2 to acc.
__device__ __forceinline__ float update_coord(float x, int32_t S, double c, double& acc) {
  const double xo = (double)x;
  const double prod = c * (double)S;
  const float xn = (float)(xo - prod);
  const double delta = (double)xn - xo;
  acc = __builtin_fma(delta, delta, acc);
  return xn;
}

__device__ __forceinline__ vf4 update_quad(vf4 xv, vi4 S, double c, double& acc) {
  vf4 xn;
  xn.x = update_coord(xv.x, S.x, c, acc);
  xn.y = update_coord(xv.y, S.y, c, acc);
  xn.z = update_coord(xv.z, S.z, c, acc);
  xn.w = update_coord(xv.w, S.w, c, acc);
  return xn;
}

__device__ __forceinline__ double decode_constant(double eta, uint32_t n, float alpha) {
  return eta / ((double)n * (double)alpha);
}

// Momentum / weight-decay form of a6 (PyTorch's SGD rule, the optimizer of Section 5's
// experiments), fp64 with every operation rounded on its own, state stored in fp32:
//   g~ = cg S (cg = 1/(n alpha));  dd = g~ + wd x;  m' = fl32(mu m + dd);  x' = fl32(x - eta m').
struct MomentumRule {
  double cg, eta, mu, wd;
};

__device__ __forceinline__ float momentum_coord(float x, float& m, int32_t S,
                                                const MomentumRule& u, double& acc) {
  const double xo = (double)x;
  const double gt = u.cg * (double)S;
  const double decay = u.wd * xo;
  const double dd = gt + decay;
  const double carried = u.mu * (double)m;
  const float mn = (float)(carried + dd);
  const double stepv = u.eta * (double)mn;
  const float xn = (float)(xo - stepv);
  const double delta = (double)xn - xo;
  acc = __builtin_fma(delta, delta, acc);
  m = mn;
  return xn;
}

__device__ __forceinline__ vf4 momentum_quad(vf4 xv, vf4& mv, vi4 S, const MomentumRule& u,
                                             double& acc) {
  vf4 xn;
  float m0 = mv.x, m1 = mv.y, m2 = mv.z, m3 = mv.w;
  xn.x = momentum_coord(xv.x, m0, S.x, u, acc);
  xn.y = momentum_coord(xv.y, m1, S.y, u, acc);
  xn.z = momentum_coord(xv.z, m2, S.z, u, acc);
  xn.w = momentum_coord(xv.w, m3, S.w, u, acc);
  mv = vf4{m0, m1, m2, m3};
  return xn;
}

// ------------------------------------------------------------------ a8
// Section 4.1 (Proposition 2) for one block, Algorithm 2 otherwise; fp64, in the
// operation order written in the public header.
__device__ __forceinline__ void apply_alpha_rule(const AlphaRule& rule, uint32_t B, uint32_t n,
                                                 uint64_t d, uint32_t l, double norm_sq) {
  const double keep = rule.beta * rule.r[l];
  const double fresh = (1.0 - rule.beta) * norm_sq;
  const double rl = keep + fresh;
  rule.r[l] = rl;
  double alpha;
  if (B == 1) {
    const double den = 2.0 * (double)n * rl / (rule.eta * rule.eta) + rule.eps * rule.eps;
    alpha = sqrt((double)d) / sqrt(den);
  } else {
    const double dl = (double)(rule.block_offsets[l + 1] - rule.block_offsets[l]);
    const double den =
        2.0 * (double)n * rl + rule.eta * rule.eta * (dl / (double)d) * rule.eps * rule.eps;
    alpha = rule.eta * sqrt(dl) / sqrt(den);
  }
  rule.alpha_out[l] = (float)alpha;
}

// ------------------------------------------------------------------ reductions behind a sweep
// Clip counts of this workgroup -> its flag and, only when some are non-zero, its column
// of the [worker][workgroup] count table plus the launch-wide hint (this launch's id)
// that tells the final-sum kernel to look at the table at all.
__device__ __forceinline__ void publish_sat(const Finish& f, const ReduceLds& lds, uint32_t wg) {
  bool any = false;
  for (uint32_t i = 0; i < f.n; ++i) any |= lds.sat[i] != 0ull;
  f.sat_any[wg] = any ? 1u : 0u;
  if (any) {
    for (uint32_t i = 0; i < f.n; ++i) f.sat_rows[(uint64_t)i * f.workgroups + wg] = lds.sat[i];
    *f.sat_hint = f.launch_id;      // every writer stores the same value
  }
}

// Sum of partial[t0, t1) by the whole workgroup in a fixed order (valid in thread 0).
// Eight independent loads in flight per lane: these kernels are pure latency.
__device__ __forceinline__ double ordered_sum(const double* partial, uint32_t t0, uint32_t t1,
                                              ReduceLds& lds) {
  double acc = 0.0;
  uint32_t t = t0 + threadIdx.x;
  for (; t + 7u * kThreads < t1; t += 8u * kThreads) {
    double v[8];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) v[u] = partial[t + u * kThreads];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) acc += v[u];
  }
  for (; t < t1; t += kThreads) acc += partial[t];
  return block_sum(acc, lds, 0);
}

// Maximum of big[t0, t1) by the whole workgroup (valid in thread 0).
__device__ __forceinline__ uint32_t range_max(const uint32_t* big, uint32_t t0, uint32_t t1,
                                              ReduceLds& lds) {
  uint32_t best = 0u;
  uint32_t t = t0 + threadIdx.x;
  for (; t + 7u * kThreads < t1; t += 8u * kThreads) {
    uint32_t v[8];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) v[u] = big[t + u * kThreads];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) best = max(best, v[u]);
  }
  for (; t < t1; t += kThreads) best = max(best, big[t]);
  return block_max(best, lds, 0);
}

// First level for very long partial lists (one block only): workgroup c sums chunk c of the
// norm partials (if any) and takes the maximum of chunk c of the largest-|S| partials (if any).
__global__ __launch_bounds__(kThreads) void k_finish_chunks(const double* partial, uint32_t count,
                                                            uint32_t chunk, double* mid,
                                                            const uint32_t* big, uint32_t* big_mid) {
  __shared__ ReduceLds lds;
  const uint32_t t0 = blockIdx.x * chunk;
  const uint32_t t1 = (count - t0 < chunk) ? count : t0 + chunk;
  if (partial != nullptr) {
    const double total = ordered_sum(partial, t0, t1, lds);
    if (threadIdx.x == 0) mid[blockIdx.x] = total;
  }
  if (big != nullptr) {
    const uint32_t best = range_max(big, t0, t1, lds);
    if (threadIdx.x == 0) big_mid[blockIdx.x] = best;
  }
}

// Workgroups [0, norm_blocks) sum the norm partials of one block each in a fixed order and
// apply the optional alpha rule to it (WITH_NORM), and take the block's largest |S_j| (if
// asked for); the n workgroups after them total one worker's clip
// counts each (reading the table only if this launch's id is in the hint word, i.e. if
// something clipped; a stale or uninitialised hint can at worst cause a needless read).
template <bool WITH_NORM, bool WITH_SAT>
__global__ __launch_bounds__(kThreads) void k_finish(const Finish f) {
  __shared__ ReduceLds lds;
  const uint32_t tid = threadIdx.x;
  const uint32_t norm_blocks = (WITH_NORM || f.big_out != nullptr) ? f.B : 0u;
  if (blockIdx.x < norm_blocks) {
    const uint32_t l = blockIdx.x;
    const uint32_t t0 = (f.B == 1) ? 0u : f.tile_prefix[l];
    const uint32_t t1 = (f.B == 1) ? f.num_tiles : f.tile_prefix[l + 1];
    if (WITH_NORM) {
      const double total = ordered_sum(f.norm_partial, t0, t1, lds);
      if (tid == 0) {
        f.norm_sq_out[l] = total;
        if (f.rule.r != nullptr) apply_alpha_rule(f.rule, f.B, f.n_workers, f.d, l, total);
      }
    }
    if (f.big_out != nullptr) {
      const uint32_t best = range_max(f.big_partial, t0, t1, lds);
      if (tid == 0) f.big_out[l] = best;
    }
    return;
  }
  if (WITH_SAT) {
    const uint32_t i = blockIdx.x - norm_blocks;           // worker
    if (tid == 0) lds.sat[0] = 0ull;
    __syncthreads();
    if (*f.sat_hint == f.launch_id) {
      const uint64_t* row = f.sat_rows + (uint64_t)i * f.workgroups;
      unsigned long long acc = 0ull;
      uint32_t g = tid;
      for (; g + 7u * kThreads < f.workgroups; g += 8u * kThreads) {
        uint32_t flag[8];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) flag[u] = f.sat_any[g + u * kThreads];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u)
          if (flag[u] != 0u) acc += row[g + u * kThreads];
      }
      for (; g < f.workgroups; g += kThreads)
        if (f.sat_any[g] != 0u) acc += row[g];
      if (acc != 0ull) atomicAdd(&lds.sat[0], acc);
    }
    __syncthreads();
    if (tid == 0) f.sat_count[i] = lds.sat[0];
  }
}

// Clip counts of the per-worker compress kernel: workgroup i sums row i.
__global__ __launch_bounds__(kThreads) void k_finish_rows(const uint64_t* rows, uint32_t row_len,
                                                          uint64_t* sat_count) {
  __shared__ unsigned long long total;
  if (threadIdx.x == 0) total = 0ull;
  __syncthreads();
  const uint64_t* row = rows + (uint64_t)blockIdx.x * row_len;
  unsigned long long acc = 0ull;
  uint32_t g = threadIdx.x;
  for (; g + 7u * kThreads < row_len; g += 8u * kThreads) {     // eight loads in flight: pure latency
    uint64_t v[8];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) v[u] = row[g + u * kThreads];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) acc += v[u];
  }
  for (; g < row_len; g += kThreads) acc += row[g];
  if (acc != 0ull) atomicAdd(&total, acc);
  __syncthreads();
  if (threadIdx.x == 0) sat_count[blockIdx.x] = total;
}

__device__ __forceinline__ void zero_sat(ReduceLds& lds) {
  if (threadIdx.x < INTSGD_MAX_WORKERS) lds.sat[threadIdx.x] = 0ull;
  __syncthreads();
}

// ================================================================== F3 (a1-a7) and F1 (a1-a4)
struct AggregateArgs {
  TileMap tm;
  RoundSpec rs;
  uint32_t n;
  const float* alpha;
  double eta;            // F3
  float* x;              // F3
  int32_t* sum_out;      // F1
  float* m;              // F3 with momentum
  double mu, wd;         // F3 with momentum
  uint64_t keep_quads;   // F3, x beyond the last-level cache: quads [0, keep_quads) are kept in it
  Finish fin;
  WorkerPtrs grads;
};

// LARGEST: also track the largest |S_j| of the tile.  A template parameter, not a run-time flag:
// the randomized sweep runs close to its vector-ALU ceiling, and the flag's branch and registers
// cost it 1-2 % even when nothing is asked for.
template <int ROUND, bool FUSED, bool MOMENTUM, int XSTORE, bool LARGEST>
struct AggregateOp {
  const AggregateArgs& a;
  ReduceLds& lds;
  float alpha;
  double c, acc;
  uint64_t q0;
  uint32_t nq;
  LaneMask any;                 // lanes of this wavefront that clipped somewhere in the tile body
  Extremes ext;                 // of the aggregates this thread formed in the tile (if asked for)
  static constexpr bool want_largest = LARGEST;
  // Randomized rounding takes the fast path (no clamp, no clip test per coordinate) and
  // redoes, counting as it goes, the rare quad of a wavefront in which something may clip.
  static constexpr bool kCountInline = ROUND == INTSGD_ROUND_STOCHASTIC;
  __amdgpu_buffer_rsrc_t out;   // x (F3) or the aggregate (F1) of this tile body
  __amdgpu_buffer_rsrc_t mom;   // momentum buffer of this tile body
  MomentumRule rule;
  bool keep;                    // this tile's part of x (and m) is to stay in the last-level cache

  __device__ __forceinline__ AggregateOp(const AggregateArgs& args, ReduceLds& l)
      : a(args), lds(l), alpha(0.f), c(0.0), acc(0.0), q0(0), nq(0), any(0ull),
        ext(extremes_init()) {}
  __device__ __forceinline__ void begin_tile(uint32_t blk) {
    alpha = a.alpha[blk];
    any = 0ull;
    ext = extremes_init();
    if (FUSED && !MOMENTUM) c = decode_constant(a.eta, a.n, alpha);
    if (MOMENTUM) rule = MomentumRule{1.0 / ((double)a.n * (double)alpha), a.eta, a.mu, a.wd};
    acc = 0.0;
  }
  __device__ __forceinline__ void scalar(uint64_t j) {
    const int32_t S = aggregate_scalar<ROUND>(a.grads, a.n, j, alpha, a.rs, lds.sat);
    if (want_largest) note(ext, S);
    if (MOMENTUM) {
      float mj = a.m[j];
      a.x[j] = momentum_coord(a.x[j], mj, S, rule, acc);
      a.m[j] = mj;
    } else if (FUSED) {
      a.x[j] = update_coord(a.x[j], S, c, acc);
    } else {
      a.sum_out[j] = S;
    }
  }
  __device__ __forceinline__ void begin_body(uint64_t first_quad, uint32_t quads) {
    q0 = first_quad;
    nq = quads;
    out = FUSED ? make_stream((vf4*)a.x + q0, nq * 16u) : make_stream((vi4*)a.sum_out + q0, nq * 16u);
    if (MOMENTUM) mom = make_stream((vf4*)a.m + q0, nq * 16u);
    keep = q0 + nq <= a.keep_quads;
  }
  // XL / XS: cache policies of this tile's x (and m) loads and stores.
  template <int XL, int XS>
  __device__ __forceinline__ void quad_with(uint32_t ql) {
    vf4 xv = vf4{0.f, 0.f, 0.f, 0.f}, mv = vf4{0.f, 0.f, 0.f, 0.f};
    if (FUSED) xv = as_f(load128<XL>(out, ql * 16u));
    if (MOMENTUM) mv = as_f(load128<XL>(mom, ql * 16u));
    vi4 S;
    if (ROUND == INTSGD_ROUND_STOCHASTIC && INTSGD_RANDOM_FAST_PATH) {
      LaneMask redo;
      S = aggregate_quad_fast(a.grads, a.n, q0, nq, ql, alpha, a.rs, redo);
      if (redo != 0ull)     // wave-uniform and rare: the exact path, which also counts per worker
        S = aggregate_quad<ROUND, true>(a.grads, a.n, q0, nq, ql, alpha, a.rs, lds.sat, any);
    } else if (ROUND == INTSGD_ROUND_STOCHASTIC) {
      S = aggregate_quad<ROUND, true>(a.grads, a.n, q0, nq, ql, alpha, a.rs, lds.sat, any);
    } else {
      S = aggregate_quad<ROUND, false>(a.grads, a.n, q0, nq, ql, alpha, a.rs, lds.sat, any);
    }
    if (want_largest) note(ext, S);
    if (MOMENTUM) {
      const vf4 xn = momentum_quad(xv, mv, S, rule, acc);
      store128<XS>(mom, ql * 16u, as_u(mv));
      store128<XS>(out, ql * 16u, as_u(xn));
    } else if (FUSED) {
      store128<XS>(out, ql * 16u, as_u(update_quad(xv, S, c, acc)));
    } else {
      store128<XS>(out, ql * 16u, as_u(S));
    }
  }
  // An x that fits the last-level cache stays there from step to step by itself.  Of a larger
  // one a prefix is kept: its tiles use the allocating policies, all other tiles read and
  // write x non-temporally so that they do not push the prefix out.
  __device__ __forceinline__ void quad(uint32_t ql) {
    if (XSTORE == kStreamOut && !(FUSED && keep)) quad_with<kNonTemporal, kStreamOut>(ql);
    else quad_with<INTSGD_X_LOAD_POLICY, kWriteThrough>(ql);
  }
  __device__ __forceinline__ void end_tile(uint32_t t, uint32_t iter) {
    if (!kCountInline && any != 0ull) {   // rare: something clipped; count it per worker
      LaneMask unused = 0ull;
      for (uint32_t ql = threadIdx.x; ql < nq; ql += kThreads)
        (void)aggregate_quad<ROUND, true>(a.grads, a.n, q0, nq, ql, alpha, a.rs, lds.sat, unused);
    }
    if (FUSED && want_largest) {
      double total;
      uint32_t best;
      block_sum_and_max(acc, magnitude(ext), lds, iter & 1u, total, best);
      if (threadIdx.x == 0) {
        a.fin.norm_partial[t] = total;
        a.fin.big_partial[t] = best;
      }
    } else if (FUSED) {
      const double total = block_sum(acc, lds, iter & 1u);
      if (threadIdx.x == 0) a.fin.norm_partial[t] = total;
    } else if (want_largest) {
      const uint32_t best = block_max(magnitude(ext), lds, iter & 1u);
      if (threadIdx.x == 0) a.fin.big_partial[t] = best;
    }
  }
};

// XSTORE: cache policy of the x / m (or S) stores, chosen by the launcher from the vector's size.
template <int ROUND, bool FUSED, bool MOMENTUM, int XSTORE, bool LARGEST>
__global__ __launch_bounds__(kThreads) void k_aggregate(const AggregateArgs a) {
  __shared__ ReduceLds lds;
  zero_sat(lds);
  AggregateOp<ROUND, FUSED, MOMENTUM, XSTORE, LARGEST> op(a, lds);
  drive_tiles(a.tm, op);
  __syncthreads();
  if (threadIdx.x == 0) publish_sat(a.fin, lds, blockIdx.x);
}

// ================================================================== F3 (a1-a7) in two phases
// One block only, one persistent workgroup of 1024 threads per CU.  The vector is cut into
// rounds of grid x 1024 x Q quads.  Within a round, iteration k of workgroup b covers the
// 1024-quad slab (k * grid + b), so at any moment the chip reads one contiguous window of
// every stream (as the tile sweep does; giving each workgroup a contiguous chunk instead
// made the rate depend on the chunk stride, HBM channel conflicts).  Phase A reads nothing
// but the n gradient streams and leaves the integer sums of the thread's Q quads in
// registers; phase B reads, updates and writes x (and the momentum buffer) for the same
// quads.  All CUs start together and move at about the same rate, so the chip alternates
// between a read-only stream and a short read-modify-write burst instead of mixing the
// two.  While x fits the memory-side cache (d up to about 50 M) the burst never reaches
// HBM and the sweep runs at 83-84 % of peak against 77-79 % for the tile sweep; beyond
// that size the two forms are within 1-3 % of each other.
struct PhasedArgs {
  RoundSpec rs;
  uint32_t n;
  const float* alpha;
  double eta;
  float* x;
  float* m;
  double mu, wd;
  int32_t* sum_out;      // kPhasedSumOnly
  uint64_t d;
  uint64_t keep_quads;   // quads [0, keep_quads) of x (and m) are kept in the last-level cache
  Finish fin;
  WorkerPtrs grads;
};

constexpr int kPhasedSumOnly = 0;    // F1: phase B writes the integer sums
constexpr int kPhasedUpdate = 1;     // F3
constexpr int kPhasedMomentum = 2;   // F3 with the momentum / weight-decay update

// Phase B for one quad: read, update and write x (and m) with the given cache policies.
template <bool MOMENTUM, int XL, int XS>
__device__ __forceinline__ void update_in_place(__amdgpu_buffer_rsrc_t out, __amdgpu_buffer_rsrc_t mom,
                                                uint32_t off, const vi4& S, double c,
                                                const MomentumRule& rule, double& acc) {
  const vf4 xv = as_f(load128<XL>(out, off));
  if (MOMENTUM) {
    vf4 mv = as_f(load128<XL>(mom, off));
    const vf4 xn = momentum_quad(xv, mv, S, rule, acc);
    store128<XS>(mom, off, as_u(mv));
    store128<XS>(out, off, as_u(xn));
  } else {
    store128<XS>(out, off, as_u(update_quad(xv, S, c, acc)));
  }
}

template <int ROUND, int MODE>
__global__ __launch_bounds__(kPhasedThreads) void k_aggregate_phased(const PhasedArgs a) {
  constexpr uint32_t kPhasedQuads = phased_quads(ROUND);
  constexpr bool MOMENTUM = MODE == kPhasedMomentum;
  __shared__ ReduceLds lds;
  zero_sat(lds);
  const uint32_t tid = threadIdx.x;
  const float alpha = a.alpha[0];
  const double c = decode_constant(a.eta, a.n, alpha);
  const MomentumRule rule{1.0 / ((double)a.n * (double)alpha), a.eta, a.mu, a.wd};
  const uint64_t nquads = a.d >> 2;
  const uint32_t slab_row = gridDim.x * kPhasedThreads;           // quads per iteration k, chip-wide
  const uint64_t per_round = (uint64_t)slab_row * kPhasedQuads;
  double acc = 0.0;
  const bool want_largest = a.fin.big_out != nullptr;      // wave-uniform
  Extremes ext = extremes_init();
  for (uint64_t r0 = 0; r0 < nquads; r0 += per_round) {
    const uint64_t rest = nquads - r0;
    const uint32_t nq = rest < per_round ? (uint32_t)rest : (uint32_t)per_round;
    // phase A: lanes past the round read zeros (the descriptors end at nq) and add 0
    vi4 S[kPhasedQuads];
    LaneMask any = 0ull;
#pragma clang loop unroll(full)
    for (uint32_t k = 0; k < kPhasedQuads; ++k) {
      S[k] = vi4{0, 0, 0, 0};
      if (k * slab_row < nq)
        S[k] = aggregate_quad<ROUND, false>(a.grads, a.n, r0, nq,
                                            (k * gridDim.x + blockIdx.x) * kPhasedThreads + tid,
                                            alpha, a.rs, lds.sat, any);
    }
    if (want_largest) {           // lanes past the round hold zeros
#pragma clang loop unroll(full)
      for (uint32_t k = 0; k < kPhasedQuads; ++k) note(ext, S[k]);
    }
    if (any != 0ull) {            // rare: something clipped in this wavefront's quads
      // Counted per worker here.  A lane past the round scales its zeros by 0 instead of
      // alpha: with a non-finite alpha, 0 * alpha is a NaN and would be counted (in the pass
      // above it can at most bring a wavefront here for nothing).
      LaneMask unused = 0ull;
#pragma clang loop unroll(disable)
      for (uint32_t k = 0; k * slab_row < nq; ++k) {
        const uint32_t ql = (k * gridDim.x + blockIdx.x) * kPhasedThreads + tid;
        (void)aggregate_quad<ROUND, true>(a.grads, a.n, r0, nq, ql, ql < nq ? alpha : 0.f, a.rs,
                                          lds.sat, unused);
      }
    }
    __syncthreads();
    // phase B: stores past the round are dropped by the descriptor
    const __amdgpu_buffer_rsrc_t out = (MODE == kPhasedSumOnly)
                                           ? make_stream((vi4*)a.sum_out + r0, nq * 16u)
                                           : make_stream((vf4*)a.x + r0, nq * 16u);
    const __amdgpu_buffer_rsrc_t mom = MOMENTUM ? make_stream((vf4*)a.m + r0, nq * 16u) : out;
#pragma clang loop unroll(full)
    for (uint32_t k = 0; k < kPhasedQuads; ++k) {
      if (k * slab_row < nq) {
        const uint32_t slab = (k * gridDim.x + blockIdx.x) * kPhasedThreads;   // of this workgroup
        const uint32_t off = (slab + tid) * 16u;
        if (MODE == kPhasedSumOnly) {       // sums that fit the cache are left there for F2
          if (a.keep_quads != 0) store128<kWriteThrough>(out, off, as_u(S[k]));
          else store128<kStreamOut>(out, off, as_u(S[k]));
        } else if (r0 + slab + kPhasedThreads <= a.keep_quads) {
          update_in_place<MOMENTUM, INTSGD_X_LOAD_POLICY, INTSGD_X_STORE_POLICY>(out, mom, off, S[k], c,
                                                                                 rule, acc);
        } else {     // the part of a large x that is streamed past the cache-resident prefix
          update_in_place<MOMENTUM, kNonTemporal, kStreamOut>(out, mom, off, S[k], c, rule, acc);
        }
      }
    }
    __syncthreads();
  }
  if (blockIdx.x == 0 && tid < (uint32_t)(a.d & 3u)) {      // the d mod 4 coordinates after the last quad
    const uint64_t j = (a.d & ~(uint64_t)3) + tid;
    const int32_t Sj = aggregate_scalar<ROUND>(a.grads, a.n, j, alpha, a.rs, lds.sat);
    if (want_largest) note(ext, Sj);
    if (MODE == kPhasedSumOnly) {
      a.sum_out[j] = Sj;
    } else if (MOMENTUM) {
      float mj = a.m[j];
      a.x[j] = momentum_coord(a.x[j], mj, Sj, rule, acc);
      a.m[j] = mj;
    } else {
      a.x[j] = update_coord(a.x[j], Sj, c, acc);
    }
  }
  const double total = block_sum(acc, lds, 0);
  uint32_t best = 0u;
  if (want_largest) best = block_max(magnitude(ext), lds, 0);
  if (tid == 0) {
    if (MODE != kPhasedSumOnly) a.fin.norm_partial[blockIdx.x] = total;
    if (want_largest) a.fin.big_partial[blockIdx.x] = best;
    publish_sat(a.fin, lds, blockIdx.x);
  }
}

// ================================================================== IntDIANA (Algorithm 3) in one sweep
// Per worker: Q_i = Int(alpha (g_i - h_i)) clipped, h_i <- h_i + Q_i / alpha; then
// g~ = h + S/(n alpha), x <- x - eta g~, h <- g~.  fp32 for the difference and the
// scale, fp64 (each operation rounded on its own) for the shifts and the update.
struct DianaArgs {
  TileMap tm;
  RoundSpec rs;
  uint32_t n;
  const float* alpha;
  double eta;
  float* x;
  float* h;              // global shift, in/out
  Finish fin;
  WorkerPtrs grads;
  WorkerOutPtrs h_local; // n local shifts, in/out
};

__device__ __forceinline__ float shift_local(float h, int32_t q, double inv_alpha) {
  const double moved = (double)q * inv_alpha;
  return (float)((double)h + moved);
}

__device__ __forceinline__ float diana_coord(float x, float& h, int32_t S, double cg, double eta,
                                             double& acc) {
  const double xo = (double)x;
  const double ghat = cg * (double)S;
  const double gt = (double)h + ghat;
  const double stepv = eta * gt;
  const float xn = (float)(xo - stepv);
  h = (float)gt;
  const double delta = (double)xn - xo;
  acc = __builtin_fma(delta, delta, acc);
  return xn;
}

template <int ROUND>
struct DianaOp {
  const DianaArgs& a;
  ReduceLds& lds;
  float alpha;
  double inv_alpha, cg, acc;
  uint64_t q0;
  uint32_t nq;
  __amdgpu_buffer_rsrc_t x_s, h_s;
  Extremes ext;                 // of the aggregates this thread formed in the tile (if asked for)
  const bool want_largest;      // wave-uniform

  __device__ __forceinline__ DianaOp(const DianaArgs& args, ReduceLds& l)
      : a(args), lds(l), alpha(0.f), inv_alpha(0.0), cg(0.0), acc(0.0), q0(0), nq(0),
        ext(extremes_init()), want_largest(args.fin.big_out != nullptr) {}
  __device__ __forceinline__ void begin_tile(uint32_t blk) {
    alpha = a.alpha[blk];
    inv_alpha = 1.0 / (double)alpha;
    cg = 1.0 / ((double)a.n * (double)alpha);
    acc = 0.0;
    ext = extremes_init();
  }
  __device__ __forceinline__ void scalar(uint64_t j) {
    int32_t S = 0;
    for (uint32_t i = 0; i < a.n; ++i) {
      float* hl = (float*)a.h_local.p[i];
      const float hv = hl[j];
      const float delta = ((const float*)a.grads.p[i])[j] - hv;
      uint32_t word = 0;
      if (ROUND == INTSGD_ROUND_STOCHASTIC) {
        const uint64_t quad = j >> 2;
        const vu4 rw = philox4x32_10((uint32_t)quad, (uint32_t)(quad >> 32), i, a.rs.step,
                                     a.rs.key0, a.rs.key1);
        word = pick_word(rw, (uint32_t)(j & 3));
      }
      LaneMask sat;
      const int32_t q = round_clip<ROUND>(alpha * delta, word, a.rs, sat);
      if (lane_in(sat)) atomicAdd(&lds.sat[i], 1ull);
      hl[j] = shift_local(hv, q, inv_alpha);
      S += q;
    }
    if (want_largest) note(ext, S);
    float hj = a.h[j];
    a.x[j] = diana_coord(a.x[j], hj, S, cg, a.eta, acc);
    a.h[j] = hj;
  }
  __device__ __forceinline__ void begin_body(uint64_t first_quad, uint32_t quads) {
    q0 = first_quad;
    nq = quads;
    x_s = make_stream((vf4*)a.x + q0, nq * 16u);
    h_s = make_stream((vf4*)a.h + q0, nq * 16u);
  }
  template <int W>
  __device__ __forceinline__ void workers(uint32_t i0, uint32_t ql, vi4& S) {
    vf4 g[W], hl[W];
    __amdgpu_buffer_rsrc_t hs[W];
#pragma unroll
    for (int w = 0; w < W; ++w) {
      const __amdgpu_buffer_rsrc_t gs = make_stream((const vf4*)a.grads.p[i0 + w] + q0, nq * 16u);
      hs[w] = make_stream((vf4*)a.h_local.p[i0 + w] + q0, nq * 16u);
      g[w] = as_f(load128<INTSGD_GRAD_LOAD_POLICY>(gs, ql * 16u));
      hl[w] = as_f(load128<INTSGD_GRAD_LOAD_POLICY>(hs[w], ql * 16u));
    }
    const uint64_t quad = q0 + ql;
#pragma unroll
    for (int w = 0; w < W; ++w) {
      vu4 word = vu4{0u, 0u, 0u, 0u};
      if (ROUND == INTSGD_ROUND_STOCHASTIC)
        word = philox4x32_10((uint32_t)quad, (uint32_t)(quad >> 32), i0 + w, a.rs.step, a.rs.key0,
                             a.rs.key1);
      const vf4 t = vf4{alpha * (g[w].x - hl[w].x), alpha * (g[w].y - hl[w].y),
                        alpha * (g[w].z - hl[w].z), alpha * (g[w].w - hl[w].w)};
      vi4 q = vi4{0, 0, 0, 0};
      LaneMask redo = ~0ull;
      if (ROUND == INTSGD_ROUND_STOCHASTIC && INTSGD_RANDOM_FAST_PATH) {
        // fast path: no clamp, no clip test; redone below if something may clip or is not finite
        int32_t q0i = 0, q1i = 0, q2i = 0, q3i = 0;
        round_random_add(t.x, word.x, q0i);
        round_random_add(t.y, word.y, q1i);
        round_random_add(t.z, word.z, q2i);
        round_random_add(t.w, word.w, q3i);
        q = vi4{q0i, q1i, q2i, q3i};
        RangeWatch watched = range_watch_init();
        watch(watched, t);
        redo = out_of_fast_range(watched, a.rs);
      }
      if (redo != 0ull) {         // nearest-even always; randomized: wave-uniform and rare
        LaneMask s0, s1, s2, s3;
        q.x = round_clip<ROUND>(t.x, word.x, a.rs, s0);
        q.y = round_clip<ROUND>(t.y, word.y, a.rs, s1);
        q.z = round_clip<ROUND>(t.z, word.z, a.rs, s2);
        q.w = round_clip<ROUND>(t.w, word.w, a.rs, s3);
        const uint32_t cnt = count_lanes(s0, s1, s2, s3);
        if (cnt != 0 && (threadIdx.x & 63u) == 0)
          atomicAdd(&lds.sat[i0 + w], (unsigned long long)cnt);
      }
      const vf4 hn = vf4{shift_local(hl[w].x, q.x, inv_alpha), shift_local(hl[w].y, q.y, inv_alpha),
                         shift_local(hl[w].z, q.z, inv_alpha), shift_local(hl[w].w, q.w, inv_alpha)};
      store128<kNonTemporal>(hs[w], ql * 16u, as_u(hn));      // n d floats: never cache resident
      S += q;
    }
  }
  __device__ __forceinline__ void quad(uint32_t ql) {
    const vf4 xv = as_f(load128<INTSGD_X_LOAD_POLICY>(x_s, ql * 16u));
    vf4 hv = as_f(load128<INTSGD_X_LOAD_POLICY>(h_s, ql * 16u));
    vi4 S = vi4{0, 0, 0, 0};
    uint32_t i = 0;
    for (; i + 4 <= a.n; i += 4) workers<4>(i, ql, S);
    if (a.n - i >= 2) { workers<2>(i, ql, S); i += 2; }
    if (a.n - i >= 1) workers<1>(i, ql, S);
    if (want_largest) note(ext, S);
    vf4 xn;
    float h0 = hv.x, h1 = hv.y, h2 = hv.z, h3 = hv.w;
    xn.x = diana_coord(xv.x, h0, S.x, cg, a.eta, acc);
    xn.y = diana_coord(xv.y, h1, S.y, cg, a.eta, acc);
    xn.z = diana_coord(xv.z, h2, S.z, cg, a.eta, acc);
    xn.w = diana_coord(xv.w, h3, S.w, cg, a.eta, acc);
    store128<kNonTemporal>(h_s, ql * 16u, as_u(vf4{h0, h1, h2, h3}));
    store128<kNonTemporal>(x_s, ql * 16u, as_u(xn));
  }
  __device__ __forceinline__ void end_tile(uint32_t t, uint32_t iter) {
    const double total = block_sum(acc, lds, iter & 1u);
    if (threadIdx.x == 0) a.fin.norm_partial[t] = total;
    if (want_largest) {
      const uint32_t best = block_max(magnitude(ext), lds, iter & 1u);
      if (threadIdx.x == 0) a.fin.big_partial[t] = best;
    }
  }
};

template <int ROUND>
__global__ __launch_bounds__(kThreads) void k_diana(const DianaArgs a) {
  __shared__ ReduceLds lds;
  zero_sat(lds);
  DianaOp<ROUND> op(a, lds);
  drive_tiles(a.tm, op);
  __syncthreads();
  if (threadIdx.x == 0) publish_sat(a.fin, lds, blockIdx.x);
}

// ================================================================== Heuristic IntSGD scaling
// Section 5.2's comparison rule (from SwitchML): alpha = (2^nb - 1)/(n 2^max_exp), where
// 2^max_exp is the smallest power of two >= the largest finite |g| of the block over all
// workers.  Pass 1 ("profiling"): per-tile maximum of the absolute bit patterns, which
// order like the values and make the reduction exact and order-free.
struct MaxAbsArgs {
  TileMap tm;
  uint32_t n;
  uint32_t* tile_max;    // one slot per tile
  WorkerPtrs grads;
};

__device__ __forceinline__ uint32_t finite_abs_bits(float v) {
  const uint32_t b = __float_as_uint(v) & 0x7FFFFFFFu;
  return b < 0x7F800000u ? b : 0u;      // Inf / NaN do not take part
}

struct MaxAbsOp {
  const MaxAbsArgs& a;
  uint32_t* lds_max;
  uint32_t best;
  uint64_t q0;
  uint32_t nq;

  __device__ __forceinline__ MaxAbsOp(const MaxAbsArgs& args, uint32_t* l)
      : a(args), lds_max(l), best(0), q0(0), nq(0) {}
  __device__ __forceinline__ void begin_tile(uint32_t) {
    best = 0;
    if (threadIdx.x == 0) *lds_max = 0u;
    __syncthreads();
  }
  __device__ __forceinline__ void scalar(uint64_t j) {
    for (uint32_t i = 0; i < a.n; ++i) best = max(best, finite_abs_bits(((const float*)a.grads.p[i])[j]));
  }
  __device__ __forceinline__ void begin_body(uint64_t first_quad, uint32_t quads) {
    q0 = first_quad;
    nq = quads;
  }
  template <int W>
  __device__ __forceinline__ void workers(uint32_t i0, uint32_t ql) {
    vf4 g[W];
#pragma unroll
    for (int w = 0; w < W; ++w) {
      const __amdgpu_buffer_rsrc_t src = make_stream((const vf4*)a.grads.p[i0 + w] + q0, nq * 16u);
      g[w] = as_f(load128<kNonTemporal>(src, ql * 16u));
    }
#pragma unroll
    for (int w = 0; w < W; ++w)
      best = max(max(best, finite_abs_bits(g[w].x)),
                 max(max(finite_abs_bits(g[w].y), finite_abs_bits(g[w].z)), finite_abs_bits(g[w].w)));
  }
  __device__ __forceinline__ void quad(uint32_t ql) {
    uint32_t i = 0;
    for (; i + 8 <= a.n; i += 8) workers<8>(i, ql);
    if (a.n - i >= 4) { workers<4>(i, ql); i += 4; }
    if (a.n - i >= 2) { workers<2>(i, ql); i += 2; }
    if (a.n - i >= 1) workers<1>(i, ql);
  }
  __device__ __forceinline__ void end_tile(uint32_t t, uint32_t) {
    if (best != 0u) atomicMax(lds_max, best);
    __syncthreads();
    if (threadIdx.x == 0) a.tile_max[t] = *lds_max;
    __syncthreads();
  }
};

__global__ __launch_bounds__(kThreads) void k_max_abs(const MaxAbsArgs a) {
  __shared__ uint32_t lds_max;
  MaxAbsOp op(a, &lds_max);
  drive_tiles(a.tm, op);
}

// Pass 2: workgroup l takes the maximum over block l's tiles and writes alpha_l.
__global__ __launch_bounds__(kThreads) void k_heuristic_alpha(const uint32_t* tile_max,
                                                              const uint32_t* tile_prefix,
                                                              uint32_t num_tiles, uint32_t B,
                                                              uint32_t n, uint32_t nb,
                                                              float* alpha_out) {
  __shared__ uint32_t lds_max;
  const uint32_t l = blockIdx.x;
  const uint32_t t0 = (B == 1) ? 0u : tile_prefix[l];
  const uint32_t t1 = (B == 1) ? num_tiles : tile_prefix[l + 1];
  if (threadIdx.x == 0) lds_max = 0u;
  __syncthreads();
  uint32_t best = 0;
  uint32_t t = t0 + threadIdx.x;
  for (; t + 7u * kThreads < t1; t += 8u * kThreads) {          // eight loads in flight: pure latency
    uint32_t v[8];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) v[u] = tile_max[t + u * kThreads];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) best = max(best, v[u]);
  }
  for (; t < t1; t += kThreads) best = max(best, tile_max[t]);
  if (best != 0u) atomicMax(&lds_max, best);
  __syncthreads();
  if (threadIdx.x != 0) return;
  const uint32_t bits = lds_max;
  double alpha = 1.0;                               // all-zero block: any alpha gives zeros
  if (bits != 0u) {
    const uint32_t field = bits >> 23, mant = bits & 0x7FFFFFu;
    int max_exp;                                    // smallest e with 2^e >= the maximum
    if (field != 0u) max_exp = (int)field - 127 + (mant != 0u ? 1 : 0);
    else max_exp = -149 + (mant > 1u ? 32 - __clz((int)(mant - 1u)) : 0);
    const double top = ldexp(1.0, (int)nb) - 1.0;
    alpha = ldexp(top / (double)n, -max_exp);
    if (alpha > 3.4028234663852886e38) alpha = 3.4028234663852886e38;   // largest finite fp32
  }
  alpha_out[l] = (float)alpha;
}

// ================================================================== a1-a3 (one worker per blockIdx.y)
struct CompressArgs {
  TileMap tm;
  RoundSpec rs;
  const float* alpha;
  uint64_t* sat_partial;   // [worker][workgroup]
  WorkerPtrs grads;
  WorkerOutPtrs q_out;
};

template <int ROUND, int WIRE>
struct CompressOp {
  const CompressArgs& a;
  ReduceLds& lds;
  uint32_t worker;
  const void* g;
  void* q;
  float alpha;
  uint64_t q0;
  __amdgpu_buffer_rsrc_t src, dst;

  __device__ __forceinline__ CompressOp(const CompressArgs& args, ReduceLds& l, uint32_t w)
      : a(args), lds(l), worker(w), g(args.grads.p[w]), q(args.q_out.p[w]), alpha(0.f), q0(0) {}
  __device__ __forceinline__ void begin_tile(uint32_t blk) { alpha = a.alpha[blk]; }
  __device__ __forceinline__ void scalar(uint64_t j) {
    LaneMask sat;
    const int32_t v = compress_scalar<ROUND>(g, j, worker, alpha, a.rs, sat);
    if (WIRE == INTSGD_WIRE_INT8) ((int8_t*)q)[j] = (int8_t)v;
    else ((int32_t*)q)[j] = v;
    if (lane_in(sat)) atomicAdd(&lds.sat[0], 1ull);
  }
  __device__ __forceinline__ void begin_body(uint64_t first_quad, uint32_t quads) {
    q0 = first_quad;
    src = make_stream((const vf4*)g + q0, quads * 16u);
    dst = (WIRE == INTSGD_WIRE_INT8) ? make_stream((uint32_t*)q + q0, quads * 4u)
                                     : make_stream((vi4*)q + q0, quads * 16u);
  }
  __device__ __forceinline__ void quad(uint32_t ql) {
    const vf4 gv = as_f(load128<INTSGD_GRAD_LOAD_POLICY>(src, ql * 16u));
    const uint64_t quad = q0 + ql;
    vu4 rw = vu4{0u, 0u, 0u, 0u};
    if (ROUND == INTSGD_ROUND_STOCHASTIC)
      rw = philox4x32_10((uint32_t)quad, (uint32_t)(quad >> 32), worker, a.rs.step, a.rs.key0,
                         a.rs.key1);
    vi4 v = vi4{0, 0, 0, 0};
    LaneMask redo = ~0ull;
    if (ROUND == INTSGD_ROUND_STOCHASTIC && INTSGD_RANDOM_FAST_PATH) {
      // fast path: no clamp, no clip test; redone below if something may clip or is not finite
      const vf4 t = vf4{alpha * gv.x, alpha * gv.y, alpha * gv.z, alpha * gv.w};
      int32_t v0 = 0, v1 = 0, v2 = 0, v3 = 0;
      round_random_add(t.x, rw.x, v0);
      round_random_add(t.y, rw.y, v1);
      round_random_add(t.z, rw.z, v2);
      round_random_add(t.w, rw.w, v3);
      v = vi4{v0, v1, v2, v3};
      RangeWatch watched = range_watch_init();
      watch(watched, t);
      redo = out_of_fast_range(watched, a.rs);
    }
    if (redo != 0ull) {           // nearest-even always; randomized: wave-uniform and rare
      LaneMask s0, s1, s2, s3;
      v.x = round_clip<ROUND>(alpha * gv.x, rw.x, a.rs, s0);
      v.y = round_clip<ROUND>(alpha * gv.y, rw.y, a.rs, s1);
      v.z = round_clip<ROUND>(alpha * gv.z, rw.z, a.rs, s2);
      v.w = round_clip<ROUND>(alpha * gv.w, rw.w, a.rs, s3);
      const uint32_t cnt = count_lanes(s0, s1, s2, s3);
      if (cnt != 0 && (threadIdx.x & 63u) == 0) atomicAdd(&lds.sat[0], (unsigned long long)cnt);
    }
    if (WIRE == INTSGD_WIRE_INT8) {
      const uint32_t packed = ((uint32_t)v.x & 0xFFu) | (((uint32_t)v.y & 0xFFu) << 8) |
                              (((uint32_t)v.z & 0xFFu) << 16) | (((uint32_t)v.w & 0xFFu) << 24);
      store32<INTSGD_X_STORE_POLICY>(dst, ql * 4u, packed);
    } else {
      // n d integers that no cache can hold until a4 reads them: written through and not
      // kept, so that nothing of them is still draining when the next kernel starts (the
      // integer sum behind this kernel: 0.313 ms -> 0.258 ms on 16 x 25.6 M)
      store128<kStreamOut>(dst, ql * 16u, as_u(v));
    }
  }
  __device__ __forceinline__ void end_tile(uint32_t, uint32_t) {}
};

template <int ROUND, int WIRE>
__global__ __launch_bounds__(kThreads) void k_compress(const CompressArgs a) {
  __shared__ ReduceLds lds;
  zero_sat(lds);
  const uint32_t worker = blockIdx.y;
  CompressOp<ROUND, WIRE> op(a, lds, worker);
  drive_tiles(a.tm, op);
  __syncthreads();
  if (threadIdx.x == 0) a.sat_partial[(uint64_t)worker * gridDim.x + blockIdx.x] = lds.sat[0];
}

// ================================================================== a4
struct IntSumArgs {
  uint64_t d;
  uint32_t n;
  uint32_t stream_out;   // the sums are too long to wait in the last-level cache for a5-a6
  int32_t* sum_out;
  WorkerPtrs q;
};

template <int WIRE>
__device__ __forceinline__ vi4 load_q4(const void* base, uint64_t quad) {
  if (WIRE == INTSGD_WIRE_INT8) {
    const uint32_t p = __builtin_nontemporal_load((const uint32_t*)base + quad);
    return vi4{(int32_t)(int8_t)(p & 0xFFu), (int32_t)(int8_t)((p >> 8) & 0xFFu),
               (int32_t)(int8_t)((p >> 16) & 0xFFu), (int32_t)(int8_t)(p >> 24)};
  }
  return __builtin_nontemporal_load((const vi4*)base + quad);
}

// Adds one 16-byte unit of a worker's integer stream to the running sums.
template <int WIRE>
__device__ __forceinline__ void add_unit(vi4 (&S)[(WIRE == INTSGD_WIRE_INT8) ? 4 : 1], const vu4& v) {
  if (WIRE == INTSGD_WIRE_INT8) {
    const uint32_t p[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      S[h].x += (int32_t)(int8_t)(p[h] & 0xFFu);
      S[h].y += (int32_t)(int8_t)((p[h] >> 8) & 0xFFu);
      S[h].z += (int32_t)(int8_t)((p[h] >> 16) & 0xFFu);
      S[h].w += (int32_t)(int8_t)(p[h] >> 24);
    }
  } else {
    S[0].x += (int32_t)v.x;
    S[0].y += (int32_t)v.y;
    S[0].z += (int32_t)v.z;
    S[0].w += (int32_t)v.w;
  }
}

// a4, tile form: workgroup b sums the 512 quads [512 b, 512 b + 512) of the n streams, eight
// loads in flight per thread (int8: one dword = four coordinates per worker and thread).
template <int WIRE>
__global__ __launch_bounds__(kThreads) void k_int_sum(const IntSumArgs a) {
  const uint64_t nq = a.d >> 2;
  const uint64_t q0 = (uint64_t)blockIdx.x * kThreads;
  if (q0 < nq) {
    const uint64_t rest = nq - q0;
    const uint32_t cnt = rest < kThreads ? (uint32_t)rest : kThreads;
    const uint32_t ql = threadIdx.x;
    vi4 S = vi4{0, 0, 0, 0};
    if (WIRE == INTSGD_WIRE_INT8) {
      if (ql < cnt)
        for (uint32_t i = 0; i < a.n; ++i) {
          const vi4 v = load_q4<WIRE>(a.q.p[i], q0 + ql);
          S.x += v.x; S.y += v.y; S.z += v.z; S.w += v.w;
        }
    } else {
      uint32_t i = 0;
      for (; i + 8 <= a.n; i += 8) {
        vu4 v[8];
#pragma unroll
        for (int w = 0; w < 8; ++w)
          v[w] = load128<kNonTemporal>(make_stream((const vu4*)a.q.p[i + w] + q0, cnt * 16u), ql * 16u);
#pragma unroll
        for (int w = 0; w < 8; ++w) {
          S.x += (int32_t)v[w].x; S.y += (int32_t)v[w].y; S.z += (int32_t)v[w].z; S.w += (int32_t)v[w].w;
        }
      }
      for (; i < a.n; ++i) {
        const vu4 v = load128<kNonTemporal>(make_stream((const vu4*)a.q.p[i] + q0, cnt * 16u), ql * 16u);
        S.x += (int32_t)v.x; S.y += (int32_t)v.y; S.z += (int32_t)v.z; S.w += (int32_t)v.w;
      }
    }
    const __amdgpu_buffer_rsrc_t out = make_stream((vi4*)a.sum_out + q0, cnt * 16u);
    if (a.stream_out) store128<kStreamOut>(out, ql * 16u, as_u(S));
    else store128<kWriteThrough>(out, ql * 16u, as_u(S));
  }
  // the d mod 4 last coordinates
  if (blockIdx.x == 0) {
    const uint64_t j = (nq << 2) + threadIdx.x;
    if (j < a.d) {
      int32_t S = 0;
      for (uint32_t i = 0; i < a.n; ++i)
        S += (WIRE == INTSGD_WIRE_INT8) ? (int32_t)((const int8_t*)a.q.p[i])[j]
                                        : ((const int32_t*)a.q.p[i])[j];
      a.sum_out[j] = S;
    }
  }
}

// a4 in two phases: per round, read the n integer streams (the sums of Q units per thread stay
// in registers), then write the sums.  A unit is 16 bytes of one worker's stream: one quad of
// int32, or 16 coordinates of int8 (whose sums go out as four 16-byte stores, transposed
// within the wavefront so that every store instruction is contiguous).
template <int WIRE>
__global__ __launch_bounds__(kPhasedThreads) void k_int_sum_phased(const IntSumArgs a) {
  constexpr uint32_t kUnitCoords = (WIRE == INTSGD_WIRE_INT8) ? 16u : 4u;
  constexpr uint32_t kUnitQuads = kUnitCoords / 4u;
  constexpr uint32_t Q = (WIRE == INTSGD_WIRE_INT8) ? 4u : 12u;      // units per thread and round
  __shared__ vi4 transpose[(WIRE == INTSGD_WIRE_INT8) ? kPhasedThreads * kUnitQuads : 1u];
  const uint32_t tid = threadIdx.x;
  const uint64_t nunits = a.d / kUnitCoords;
  const uint32_t slab_row = gridDim.x * kPhasedThreads;
  const uint64_t per_round = (uint64_t)slab_row * Q;
  for (uint64_t r0 = 0; r0 < nunits; r0 += per_round) {
    const uint64_t rest = nunits - r0;
    const uint32_t nu = rest < per_round ? (uint32_t)rest : (uint32_t)per_round;
    vi4 S[Q][kUnitQuads];
#pragma clang loop unroll(full)
    for (uint32_t k = 0; k < Q; ++k)
#pragma clang loop unroll(full)
      for (uint32_t h = 0; h < kUnitQuads; ++h) S[k][h] = vi4{0, 0, 0, 0};
#pragma clang loop unroll(full)
    for (uint32_t k = 0; k < Q; ++k) {
      if (k * slab_row < nu) {
        const uint32_t off = ((k * gridDim.x + blockIdx.x) * kPhasedThreads + tid) * 16u;
        uint32_t i = 0;
        for (; i + 8 <= a.n; i += 8) {
          vu4 v[8];
#pragma unroll
          for (int w = 0; w < 8; ++w)
            v[w] = load128<kNonTemporal>(make_stream((const vu4*)a.q.p[i + w] + r0, nu * 16u), off);
#pragma unroll
          for (int w = 0; w < 8; ++w) add_unit<WIRE>(S[k], v[w]);
        }
        for (; i < a.n; ++i)
          add_unit<WIRE>(S[k], load128<kNonTemporal>(make_stream((const vu4*)a.q.p[i] + r0, nu * 16u), off));
      }
    }
    __syncthreads();
    const __amdgpu_buffer_rsrc_t out =
        make_stream((vi4*)a.sum_out + r0 * kUnitQuads, nu * 16u * kUnitQuads);
#pragma clang loop unroll(full)
    for (uint32_t k = 0; k < Q; ++k) {
      if (k * slab_row < nu) {
        const uint32_t unit = (k * gridDim.x + blockIdx.x) * kPhasedThreads + tid;
        if (WIRE == INTSGD_WIRE_INT8) {
          // A lane holds the four quads of its 64 output bytes.  Written as they are, every store
          // instruction would touch 64 cache lines a quarter each; a wavefront-local transpose
          // through LDS makes each of the four stores one contiguous kilobyte instead.
          const uint32_t lane = tid & 63u;
          vi4* tr = transpose + (tid & ~63u) * kUnitQuads;           // this wavefront's 256 quads
#pragma clang loop unroll(full)
          for (uint32_t h = 0; h < kUnitQuads; ++h) tr[lane * kUnitQuads + h] = S[k][h];
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          const uint32_t first_quad = (unit - lane) * kUnitQuads;    // of the wavefront's 64 units
#pragma clang loop unroll(full)
          for (uint32_t h = 0; h < kUnitQuads; ++h) {
            const uint32_t off = (first_quad + h * 64u + lane) * 16u;
            if (a.stream_out) store128<kStreamOut>(out, off, as_u(tr[h * 64u + lane]));
            else store128<kWriteThrough>(out, off, as_u(tr[h * 64u + lane]));
          }
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else {
#pragma clang loop unroll(full)
          for (uint32_t h = 0; h < kUnitQuads; ++h) {
            if (a.stream_out) store128<kStreamOut>(out, (unit * kUnitQuads + h) * 16u, as_u(S[k][h]));
            else store128<kWriteThrough>(out, (unit * kUnitQuads + h) * 16u, as_u(S[k][h]));
          }
        }
      }
    }
    __syncthreads();
  }
  // the coordinates after the last whole unit
  if (blockIdx.x == 0) {
    const uint64_t j = nunits * kUnitCoords + tid;
    if (j < a.d) {
      int32_t Sj = 0;
      for (uint32_t i = 0; i < a.n; ++i)
        Sj += (WIRE == INTSGD_WIRE_INT8) ? (int32_t)((const int8_t*)a.q.p[i])[j]
                                         : ((const int32_t*)a.q.p[i])[j];
      a.sum_out[j] = Sj;
    }
  }
}

// ================================================================== a5-a6 (and F2 = a5-a7)
struct DecodeArgs {
  TileMap tm;
  uint32_t n;
  const int32_t* sum;
  const float* alpha;
  double eta;
  float* x;
  float* gtilde;         // decode_update only, may be null
  float* m;              // momentum form only
  double mu, wd;         // momentum form only
  uint64_t keep_quads;   // quads [0, keep_quads) of x (and m) are kept in the last-level cache
  Finish fin;            // F2 only
};

template <bool WITH_NORM, bool WITH_GTILDE, bool MOMENTUM>
struct DecodeOp {
  const DecodeArgs& a;
  ReduceLds& lds;
  double c, na, acc;
  __amdgpu_buffer_rsrc_t sum_s, x_s, gt_s, m_s;
  MomentumRule rule;
  bool keep;             // this tile's part of x (and m) stays in the last-level cache

  __device__ __forceinline__ DecodeOp(const DecodeArgs& args, ReduceLds& l)
      : a(args), lds(l), c(0.0), na(0.0), acc(0.0) {}
  __device__ __forceinline__ void begin_tile(uint32_t blk) {
    const float alpha = a.alpha[blk];
    na = (double)a.n * (double)alpha;
    c = decode_constant(a.eta, a.n, alpha);
    if (MOMENTUM) rule = MomentumRule{1.0 / na, a.eta, a.mu, a.wd};
    acc = 0.0;
  }
  __device__ __forceinline__ float gtilde_of(int32_t S) const { return (float)((double)S / na); }
  __device__ __forceinline__ void scalar(uint64_t j) {
    const int32_t S = a.sum[j];
    if (MOMENTUM) {
      float mj = a.m[j];
      a.x[j] = momentum_coord(a.x[j], mj, S, rule, acc);
      a.m[j] = mj;
    } else {
      a.x[j] = update_coord(a.x[j], S, c, acc);
    }
    if (WITH_GTILDE) a.gtilde[j] = gtilde_of(S);
  }
  __device__ __forceinline__ void begin_body(uint64_t q0, uint32_t quads) {
    sum_s = make_stream((const vi4*)a.sum + q0, quads * 16u);
    x_s = make_stream((vf4*)a.x + q0, quads * 16u);
    if (WITH_GTILDE) gt_s = make_stream((vf4*)a.gtilde + q0, quads * 16u);
    if (MOMENTUM) m_s = make_stream((vf4*)a.m + q0, quads * 16u);
    keep = q0 + quads <= a.keep_quads;
  }
  __device__ __forceinline__ void quad(uint32_t ql) {
    const vi4 S = as_i(load128<kNonTemporal>(sum_s, ql * 16u));
    // the cache-resident prefix of a large x, or the streamed rest (as in the fused sweeps)
    if (keep)
      update_in_place<MOMENTUM, INTSGD_X_LOAD_POLICY, INTSGD_X_STORE_POLICY>(x_s, m_s, ql * 16u, S, c,
                                                                             rule, acc);
    else
      update_in_place<MOMENTUM, kNonTemporal, kStreamOut>(x_s, m_s, ql * 16u, S, c, rule, acc);
    if (WITH_GTILDE) {
      const vf4 gt = vf4{gtilde_of(S.x), gtilde_of(S.y), gtilde_of(S.z), gtilde_of(S.w)};
      store128<kPlain>(gt_s, ql * 16u, as_u(gt));
    }
  }
  __device__ __forceinline__ void end_tile(uint32_t t, uint32_t iter) {
    if (WITH_NORM) {
      const double total = block_sum(acc, lds, iter & 1u);
      if (threadIdx.x == 0) a.fin.norm_partial[t] = total;
    }
  }
};

template <bool WITH_NORM, bool WITH_GTILDE, bool MOMENTUM>
__global__ __launch_bounds__(kThreads) void k_decode(const DecodeArgs a) {
  __shared__ ReduceLds lds;
  DecodeOp<WITH_NORM, WITH_GTILDE, MOMENTUM> op(a, lds);
  drive_tiles(a.tm, op);
}

// ================================================================== a7
struct NormArgs {
  TileMap tm;
  const float* x_new;
  const float* x_old;
  Finish fin;
};

struct NormOp {
  const NormArgs& a;
  ReduceLds& lds;
  double acc;
  __amdgpu_buffer_rsrc_t new_s, old_s;

  __device__ __forceinline__ NormOp(const NormArgs& args, ReduceLds& l) : a(args), lds(l), acc(0.0) {}
  __device__ __forceinline__ void add(float xn, float xo) {
    const double delta = (double)xn - (double)xo;
    acc = __builtin_fma(delta, delta, acc);
  }
  __device__ __forceinline__ void begin_tile(uint32_t) { acc = 0.0; }
  __device__ __forceinline__ void scalar(uint64_t j) { add(a.x_new[j], a.x_old[j]); }
  __device__ __forceinline__ void begin_body(uint64_t q0, uint32_t quads) {
    new_s = make_stream((const vf4*)a.x_new + q0, quads * 16u);
    old_s = make_stream((const vf4*)a.x_old + q0, quads * 16u);
  }
  __device__ __forceinline__ void quad(uint32_t ql) {
    const vf4 n4 = as_f(load128<kNonTemporal>(new_s, ql * 16u));
    const vf4 o4 = as_f(load128<kNonTemporal>(old_s, ql * 16u));
    add(n4.x, o4.x); add(n4.y, o4.y); add(n4.z, o4.z); add(n4.w, o4.w);
  }
  __device__ __forceinline__ void end_tile(uint32_t t, uint32_t iter) {
    const double total = block_sum(acc, lds, iter & 1u);
    if (threadIdx.x == 0) a.fin.norm_partial[t] = total;
  }
};

__global__ __launch_bounds__(kThreads) void k_update_norm(const NormArgs a) {
  __shared__ ReduceLds lds;
  NormOp op(a, lds);
  drive_tiles(a.tm, op);
}

// ================================================================== a8 on its own
__global__ __launch_bounds__(256) void k_next_alpha(const double* norm_sq, AlphaRule rule, uint32_t B,
                                                    uint32_t n, uint64_t d) {
  const uint32_t l = blockIdx.x * 256u + threadIdx.x;
  if (l < B) apply_alpha_rule(rule, B, n, d, l, norm_sq[l]);
}

inline hipError_t after_launch() { return hipGetLastError(); }

// Records the optional profiling taps around the streaming kernel of a call.
// Launches a streaming kernel.  With profiling taps pending, the two events are attached to
// the dispatch itself, so that their difference is the kernel's own duration (what a profiler
// reports) and not kernel + dispatch latency.
#define launch_sweep(ls, kernel, grid, block, lds, ...)                                          \
  do {                                                                                           \
    if ((ls).tap_start != nullptr && (ls).tap_stop != nullptr)                                   \
      hipExtLaunchKernelGGL(kernel, grid, block, lds, (ls).stream, (ls).tap_start, (ls).tap_stop, \
                            0u, __VA_ARGS__);                                                    \
    else                                                                                         \
      hipLaunchKernelGGL(kernel, grid, block, lds, (ls).stream, __VA_ARGS__);                    \
  } while (0)

// The 256 MB last-level (memory-side) cache: a state vector up to kResidentBytes is left to stay
// in it as a whole; of a larger one the first kKeepBytes are kept and the rest is streamed.
constexpr uint64_t kResidentBytes = 192ull << 20;
constexpr uint64_t kKeepBytes = 224ull << 20;

// Quads of x (and of m) that a sweep over d coordinates keeps cache-resident.
uint64_t state_keep_quads(uint64_t d, bool with_momentum) {
  const uint64_t vectors = with_momentum ? 2u : 1u;
  if (vectors * d * sizeof(float) <= kResidentBytes) return ~0ull;
  return kKeepBytes / 16u / vectors;
}

// The integer sums between F1 and F2 stay in the cache only if x fits beside them.
bool sums_stay_resident(uint64_t d) { return 2u * d * sizeof(int32_t) <= kKeepBytes; }

constexpr uint32_t kChunk = 8192;            // partials per first-level workgroup
constexpr uint32_t kTwoLevelFrom = 2 * kChunk;

hipError_t finish(hipStream_t stream, const Finish& fin_in, bool with_norm, bool with_sat) {
  Finish fin = fin_in;
  const bool with_big = fin.big_out != nullptr;
  if ((with_norm || with_big) && fin.B == 1 && fin.num_tiles > kTwoLevelFrom) {
    const uint32_t chunks = (fin.num_tiles + kChunk - 1) / kChunk;
    hipLaunchKernelGGL(k_finish_chunks, dim3(chunks), dim3(kThreads), 0, stream,
                       with_norm ? fin.norm_partial : nullptr, fin.num_tiles, kChunk, fin.norm_mid,
                       with_big ? fin.big_partial : nullptr, fin.big_mid);
    const hipError_t e = after_launch();
    if (e != hipSuccess) return e;
    fin.norm_partial = fin.norm_mid;
    fin.big_partial = fin.big_mid;
    fin.num_tiles = chunks;
  }
  const dim3 grid(((with_norm || with_big) ? fin.B : 0u) + (with_sat ? fin.n : 0u)), block(kThreads);
  if (with_norm && with_sat) hipLaunchKernelGGL((k_finish<true, true>), grid, block, 0, stream, fin);
  else if (with_norm) hipLaunchKernelGGL((k_finish<true, false>), grid, block, 0, stream, fin);
  else hipLaunchKernelGGL((k_finish<false, true>), grid, block, 0, stream, fin);
  return after_launch();
}

}  // namespace

// ------------------------------------------------------------------ launchers
hipError_t launch_compress(const TileMap& tm, const LaunchShape& ls, uint32_t n, int32_t wire,
                           const RoundSpec& rs, const WorkerPtrs& grads, const float* alpha,
                           const WorkerOutPtrs& q_out, uint64_t* sat_partial,
                           uint64_t* sat_count) {
  CompressArgs a{tm, rs, alpha, sat_partial, grads, q_out};
  const dim3 grid(ls.grid, n), block(kThreads);
  const bool random = rs.rounding == INTSGD_ROUND_STOCHASTIC;
  {
    if (wire == INTSGD_WIRE_INT8) {
      if (random) launch_sweep(ls, (k_compress<1, 8>), grid, block, ls.lds_reserve, a);
      else launch_sweep(ls, (k_compress<0, 8>), grid, block, ls.lds_reserve, a);
    } else {
      if (random) launch_sweep(ls, (k_compress<1, 32>), grid, block, ls.lds_reserve, a);
      else launch_sweep(ls, (k_compress<0, 32>), grid, block, ls.lds_reserve, a);
    }
  }
  hipError_t e = after_launch();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_finish_rows, dim3(n), dim3(kThreads), 0, ls.stream, sat_partial, ls.grid,
                     sat_count);
  return after_launch();
}

hipError_t launch_int_sum_phased(const PhasedShape& ps, const LaunchShape& ls, uint64_t d, uint32_t n,
                                 int32_t wire, const WorkerPtrs& q, int32_t* sum_out) {
  IntSumArgs a{d, n, sums_stay_resident(d) ? 0u : 1u, sum_out, q};
  const dim3 grid(ps.grid), block(kPhasedThreads);
  if (wire == INTSGD_WIRE_INT8) launch_sweep(ls, (k_int_sum_phased<8>), grid, block, 0, a);
  else launch_sweep(ls, (k_int_sum_phased<32>), grid, block, 0, a);
  return after_launch();
}

hipError_t launch_int_sum(uint64_t d, const LaunchShape& ls, uint32_t n, int32_t wire,
                          const WorkerPtrs& q, int32_t* sum_out) {
  IntSumArgs a{d, n, sums_stay_resident(d) ? 0u : 1u, sum_out, q};
  const dim3 grid(ls.grid), block(kThreads);
  if (wire == INTSGD_WIRE_INT8) launch_sweep(ls, (k_int_sum<8>), grid, block, 0, a);
  else launch_sweep(ls, (k_int_sum<32>), grid, block, 0, a);
  return after_launch();
}

hipError_t launch_decode_update(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                                const int32_t* sum, const float* alpha, double eta, float* x,
                                float* gtilde_out) {
  DecodeArgs a{tm, n, sum, alpha, eta, x, gtilde_out, nullptr, 0.0, 0.0, state_keep_quads(tm.d, false),
               Finish{}};
  const dim3 grid(ls.grid), block(kThreads);
  if (gtilde_out) launch_sweep(ls, (k_decode<false, true, false>), grid, block, 0, a);
  else launch_sweep(ls, (k_decode<false, false, false>), grid, block, 0, a);
  return after_launch();
}

hipError_t launch_update_norm(const TileMap& tm, const LaunchShape& ls, const float* x_new,
                              const float* x_old, const Finish& fin) {
  NormArgs a{tm, x_new, x_old, fin};
  {
    launch_sweep(ls, k_update_norm, dim3(ls.grid), dim3(kThreads), 0, a);
  }
  hipError_t e = after_launch();
  if (e != hipSuccess) return e;
  return finish(ls.stream, fin, true, false);
}

hipError_t launch_compress_sum(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                               const RoundSpec& rs, const WorkerPtrs& grads, const float* alpha,
                               int32_t* sum_out, const Finish& fin) {
  AggregateArgs a{tm, rs, n, alpha, 0.0, nullptr, sum_out, nullptr, 0.0, 0.0, 0, fin, grads};
  const dim3 grid(ls.grid), block(kThreads);
  const bool random = rs.rounding == INTSGD_ROUND_STOCHASTIC;
  const bool largest = fin.big_out != nullptr;
#define INTSGD_LAUNCH_F1(R, XS)                                                                        \
  do {                                                                                                 \
    if (largest) launch_sweep(ls, (k_aggregate<R, false, false, XS, true>), grid, block, ls.lds_reserve, a); \
    else launch_sweep(ls, (k_aggregate<R, false, false, XS, false>), grid, block, ls.lds_reserve, a);  \
  } while (0)
  if (sums_stay_resident(tm.d)) {
    if (random) INTSGD_LAUNCH_F1(1, kWriteThrough);
    else INTSGD_LAUNCH_F1(0, kWriteThrough);
  } else {      // streamed: the sums would only push x out of the cache
    if (random) INTSGD_LAUNCH_F1(1, kStreamOut);
    else INTSGD_LAUNCH_F1(0, kStreamOut);
  }
#undef INTSGD_LAUNCH_F1
  hipError_t e = after_launch();
  if (e != hipSuccess) return e;
  return finish(ls.stream, fin, false, true);
}

hipError_t launch_decode_update_norm(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                                     const int32_t* sum, const float* alpha, double eta, float* x,
                                     const Momentum* mom, const Finish& fin) {
  DecodeArgs a{tm, n, sum, alpha, eta, x, nullptr, mom ? mom->m : nullptr, mom ? mom->mu : 0.0,
               mom ? mom->wd : 0.0, state_keep_quads(tm.d, mom != nullptr), fin};
  {
    if (mom)
      launch_sweep(ls, (k_decode<true, false, true>), dim3(ls.grid), dim3(kThreads), 0, a);
    else
      launch_sweep(ls, (k_decode<true, false, false>), dim3(ls.grid), dim3(kThreads), 0, a);
  }
  hipError_t e = after_launch();
  if (e != hipSuccess) return e;
  return finish(ls.stream, fin, true, false);
}

hipError_t launch_step_fused(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                             const RoundSpec& rs, const WorkerPtrs& grads, const float* alpha,
                             double eta, float* x, const Momentum* mom, const Finish& fin) {
  AggregateArgs a{tm, rs, n, alpha, eta, x, nullptr, mom ? mom->m : nullptr, mom ? mom->mu : 0.0,
                  mom ? mom->wd : 0.0, 0, fin, grads};
  const dim3 grid(ls.grid), block(kThreads);
  const bool random = rs.rounding == INTSGD_ROUND_STOCHASTIC;
  // x (and m) no larger than the 256 MB last-level cache stay there from one step to the next
  // when written through.  Of a larger x a prefix of kKeepBytes is treated that way and the
  // rest is read and written non-temporally, which leaves the prefix in the cache: on
  // workload 4 (434 MB of x) 0.741 -> 0.705 ms, and the streamed part by itself is 2-3 %
  // faster with nt + sc1 stores than with plain write-through ones.
  a.keep_quads = state_keep_quads(tm.d, mom != nullptr);
  const bool big = a.keep_quads != ~0ull;
  const bool largest = fin.big_out != nullptr;
#define INTSGD_LAUNCH_AGG_L(R, M, L)                                                                   \
  do {                                                                                                 \
    if (big) launch_sweep(ls, (k_aggregate<R, true, M, kStreamOut, L>), grid, block, ls.lds_reserve, a); \
    else launch_sweep(ls, (k_aggregate<R, true, M, kWriteThrough, L>), grid, block, ls.lds_reserve, a);  \
  } while (0)
#define INTSGD_LAUNCH_AGG(R, M)              \
  do {                                       \
    if (largest) INTSGD_LAUNCH_AGG_L(R, M, true); \
    else INTSGD_LAUNCH_AGG_L(R, M, false);   \
  } while (0)
  if (mom) {
    if (random) INTSGD_LAUNCH_AGG(1, true);
    else INTSGD_LAUNCH_AGG(0, true);
  } else {
    if (random) INTSGD_LAUNCH_AGG(1, false);
    else INTSGD_LAUNCH_AGG(0, false);
  }
#undef INTSGD_LAUNCH_AGG
#undef INTSGD_LAUNCH_AGG_L
  hipError_t e = after_launch();
  if (e != hipSuccess) return e;
  return finish(ls.stream, fin, true, true);
}

hipError_t launch_step_fused_phased(const PhasedShape& ps, const LaunchShape& ls, uint64_t d,
                                    uint32_t n, const RoundSpec& rs, const WorkerPtrs& grads,
                                    const float* alpha, double eta, float* x, const Momentum* mom,
                                    const Finish& fin_in) {
  Finish fin = fin_in;
  fin.num_tiles = ps.grid;      // one norm partial and one clip-table column per workgroup
  fin.workgroups = ps.grid;
  // same rule as the tile sweep: an x beyond the last-level cache keeps a prefix in it
  const uint64_t keep_quads = state_keep_quads(d, mom != nullptr);
  PhasedArgs a{rs, n, alpha, eta, x, mom ? mom->m : nullptr, mom ? mom->mu : 0.0,
               mom ? mom->wd : 0.0, nullptr, d, keep_quads, fin, grads};
  const dim3 grid(ps.grid), block(kPhasedThreads);
  const bool random = rs.rounding == INTSGD_ROUND_STOCHASTIC;
  {
    if (mom) {
      if (random) launch_sweep(ls, (k_aggregate_phased<1, kPhasedMomentum>), grid, block, 0, a);
      else launch_sweep(ls, (k_aggregate_phased<0, kPhasedMomentum>), grid, block, 0, a);
    } else {
      if (random) launch_sweep(ls, (k_aggregate_phased<1, kPhasedUpdate>), grid, block, 0, a);
      else launch_sweep(ls, (k_aggregate_phased<0, kPhasedUpdate>), grid, block, 0, a);
    }
  }
  hipError_t e = after_launch();
  if (e != hipSuccess) return e;
  return finish(ls.stream, fin, true, true);
}

hipError_t launch_compress_sum_phased(const PhasedShape& ps, const LaunchShape& ls, uint64_t d,
                                      uint32_t n, const RoundSpec& rs, const WorkerPtrs& grads,
                                      const float* alpha, int32_t* sum_out, const Finish& fin_in) {
  Finish fin = fin_in;
  fin.num_tiles = ps.grid;
  fin.workgroups = ps.grid;
  PhasedArgs a{rs, n, alpha, 0.0, nullptr, nullptr, 0.0, 0.0, sum_out, d,
               sums_stay_resident(d) ? ~0ull : 0ull, fin, grads};
  const dim3 grid(ps.grid), block(kPhasedThreads);
  {
    if (rs.rounding == INTSGD_ROUND_STOCHASTIC)
      launch_sweep(ls, (k_aggregate_phased<1, kPhasedSumOnly>), grid, block, 0, a);
    else
      launch_sweep(ls, (k_aggregate_phased<0, kPhasedSumOnly>), grid, block, 0, a);
  }
  hipError_t e = after_launch();
  if (e != hipSuccess) return e;
  return finish(ls.stream, fin, false, true);
}

hipError_t launch_diana_step(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                             const RoundSpec& rs, const WorkerPtrs& grads,
                             const WorkerOutPtrs& h_local, const float* alpha, double eta, float* x,
                             float* h, const Finish& fin) {
  DianaArgs a{tm, rs, n, alpha, eta, x, h, fin, grads, h_local};
  const dim3 grid(ls.grid), block(kThreads);
  {
    if (rs.rounding == INTSGD_ROUND_STOCHASTIC)
      launch_sweep(ls, (k_diana<1>), grid, block, ls.lds_reserve, a);
    else
      launch_sweep(ls, (k_diana<0>), grid, block, ls.lds_reserve, a);
  }
  hipError_t e = after_launch();
  if (e != hipSuccess) return e;
  return finish(ls.stream, fin, true, true);
}

hipError_t launch_heuristic_alpha(const TileMap& tm, const LaunchShape& ls, uint32_t n, uint32_t nb,
                                  const WorkerPtrs& grads, uint32_t* tile_max,
                                  const uint32_t* tile_prefix, uint32_t B, float* alpha_out) {
  MaxAbsArgs a{tm, n, tile_max, grads};
  {
    launch_sweep(ls, k_max_abs, dim3(ls.grid), dim3(kThreads), ls.lds_reserve, a);
  }
  hipError_t e = after_launch();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_heuristic_alpha, dim3(B), dim3(kThreads), 0, ls.stream, tile_max, tile_prefix,
                     tm.num_tiles, B, n, nb, alpha_out);
  return after_launch();
}

hipError_t launch_next_alpha(hipStream_t stream, const double* norm_sq, const AlphaRule& rule,
                             uint32_t B, uint32_t n, uint64_t d) {
  const uint32_t blocks = (B + 255u) / 256u;
  hipLaunchKernelGGL(k_next_alpha, dim3(blocks), dim3(256), 0, stream, norm_sq, rule, B, n, d);
  return after_launch();
}

}  // namespace intsgd
