// Internal interface between the host side of the C ABI (intsgd_api.cpp) and the
// kernel launchers (intsgd_kernels.hip).  Not installed; not part of the ABI.
#ifndef INTSGD_INTERNAL_H_
#define INTSGD_INTERNAL_H_

#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "intsgd.h"

namespace intsgd {

// One unit of work: coordinates [start, start+len) that all lie in block blk.
struct TileEntry {
  uint64_t start;
  uint32_t len;
  uint32_t blk;
};

// How a launch maps tile indices to coordinates.  table == nullptr: one block,
// tile t covers [t*tile, min(d, (t+1)*tile)).  Otherwise table[t] (device memory).
struct TileMap {
  uint64_t d;
  uint32_t tile;
  uint32_t num_tiles;
  const TileEntry* table;
  uint32_t xcd_shift;    // 0, or log2 of the run of consecutive tiles each XCD takes (see drive_tiles)
};

// Per-worker device pointers, passed to kernels by value in the kernarg segment.
struct WorkerPtrs {
  const void* p[INTSGD_MAX_WORKERS];
};
struct WorkerOutPtrs {
  void* p[INTSGD_MAX_WORKERS];
};

// Everything the rounding stage needs besides alpha.
struct RoundSpec {
  int32_t rounding;      // intsgd_rounding
  int32_t clip;          // L
  float sat_threshold;   // smallest fp32 >= L+1: an integer-valued fp32 r is clipped iff !(|r| < it)
  uint32_t fast_limit_bits;  // bits of the largest fp32 <= L: |t| below it cannot clip whichever way t is rounded
  uint32_t key0, key1;   // lo32(seed), hi32(seed)
  uint32_t step;
};

#define INTSGD_THREADS_PER_WORKGROUP 512

struct LaunchShape {
  uint32_t grid;         // workgroups along x
  uint32_t lds_reserve;  // extra dynamic LDS per workgroup (caps workgroups per CU), heavy kernels
  hipStream_t stream;
  hipEvent_t tap_start, tap_stop;  // optional profiling taps around the streaming kernel
};

// Shape of the two-phase fused sweep: one persistent workgroup per CU.
struct PhasedShape {
  uint32_t grid;
};

// The alpha rule of step a8 on device arrays; r == nullptr means "do not apply".
struct AlphaRule {
  double* r;                      // B, in/out
  float* alpha_out;               // B
  const uint64_t* block_offsets;  // device, B+1, or null when B == 1
  double beta, eps, eta;
};

// Momentum / weight-decay form of the update: state vector and coefficients.
struct Momentum {
  float* m;      // device, d
  double mu, wd;
};

// What the final-sum kernel behind a sweep needs.
struct Finish {
  double* norm_partial;           // one slot per tile
  double* norm_mid;               // first-level sums when the tile list is very long
  const uint32_t* tile_prefix;    // device, B+1: tile range of each block; unused when B == 1
  uint32_t num_tiles;
  uint32_t B;
  double* norm_sq_out;            // B
  uint32_t workgroups;            // grid of the sweep
  uint32_t* sat_hint;             // holds launch_id if some workgroup of this launch clipped
  uint32_t launch_id;             // non-zero, different for consecutive launches
  uint32_t* sat_any;              // one flag per workgroup
  uint64_t* sat_rows;             // [worker][workgroup], written only where the flag is set
  uint32_t n;                     // workers (clip counts)
  uint64_t* sat_count;            // n
  uint32_t n_workers;             // n of the problem (alpha rule)
  uint64_t d;
  AlphaRule rule;
  uint32_t* big_partial;          // one slot per tile: largest |S_j| of the tile (used only with big_out)
  uint32_t* big_mid;              // first-level maxima when the tile list is very long
  uint32_t* big_out;              // B, or null: the largest |S_j| per block is not asked for
};

// Address, on the current device, of the library's static device scratch array of
// INTSGD_STATIC_SCRATCH_BYTES (resolved once per device, then cached).  Allocates nothing.
hipError_t static_scratch(void** ptr);

// Every launcher only enqueues; the return value is hipGetLastError() after the launch.
hipError_t launch_compress(const TileMap& tm, const LaunchShape& ls, uint32_t n, int32_t wire,
                           const RoundSpec& rs, const WorkerPtrs& grads, const float* alpha,
                           const WorkerOutPtrs& q_out, uint64_t* sat_partial,
                           uint64_t* sat_count);
hipError_t launch_int_sum(uint64_t d, const LaunchShape& ls, uint32_t n, int32_t wire,
                          const WorkerPtrs& q, int32_t* sum_out);
hipError_t launch_decode_update(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                                const int32_t* sum, const float* alpha, double eta, float* x,
                                float* gtilde_out);
hipError_t launch_update_norm(const TileMap& tm, const LaunchShape& ls, const float* x_new,
                              const float* x_old, const Finish& fin);
hipError_t launch_compress_sum(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                               const RoundSpec& rs, const WorkerPtrs& grads, const float* alpha,
                               int32_t* sum_out, const Finish& fin);
hipError_t launch_decode_update_norm(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                                     const int32_t* sum, const float* alpha, double eta, float* x,
                                     const Momentum* mom, const Finish& fin);
hipError_t launch_step_fused(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                             const RoundSpec& rs, const WorkerPtrs& grads, const float* alpha,
                             double eta, float* x, const Momentum* mom, const Finish& fin);
// Same step in the two-phase form (one block only, 16-byte aligned rows, any n).
hipError_t launch_step_fused_phased(const PhasedShape& ps, const LaunchShape& ls, uint64_t d,
                                    uint32_t n, const RoundSpec& rs, const WorkerPtrs& grads,
                                    const float* alpha, double eta, float* x, const Momentum* mom,
                                    const Finish& fin);
// F1 in the two-phase form: phase B writes the integer sums.
hipError_t launch_compress_sum_phased(const PhasedShape& ps, const LaunchShape& ls, uint64_t d,
                                      uint32_t n, const RoundSpec& rs, const WorkerPtrs& grads,
                                      const float* alpha, int32_t* sum_out, const Finish& fin);
// a4 in the two-phase form.
hipError_t launch_int_sum_phased(const PhasedShape& ps, const LaunchShape& ls, uint64_t d, uint32_t n,
                                 int32_t wire, const WorkerPtrs& q, int32_t* sum_out);
hipError_t launch_diana_step(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                             const RoundSpec& rs, const WorkerPtrs& grads,
                             const WorkerOutPtrs& h_local, const float* alpha, double eta, float* x,
                             float* h, const Finish& fin);
hipError_t launch_heuristic_alpha(const TileMap& tm, const LaunchShape& ls, uint32_t n, uint32_t nb,
                                  const WorkerPtrs& grads, uint32_t* tile_max,
                                  const uint32_t* tile_prefix, uint32_t B, float* alpha_out);
hipError_t launch_next_alpha(hipStream_t stream, const double* norm_sq, const AlphaRule& rule,
                             uint32_t B, uint32_t n, uint64_t d);

}  // namespace intsgd

#endif  // INTSGD_INTERNAL_H_
