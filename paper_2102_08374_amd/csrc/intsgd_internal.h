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
  uint32_t key0, key1;   // lo32(seed), hi32(seed)
  uint32_t step;
};

struct LaunchShape {
  uint32_t grid;         // workgroups along x
  hipStream_t stream;
};

// Every launcher only enqueues; the return value is hipGetLastError() after the launch.
hipError_t launch_compress(const TileMap& tm, const LaunchShape& ls, uint32_t n, int32_t wire,
                           const RoundSpec& rs, const WorkerPtrs& grads, const float* alpha,
                           const WorkerOutPtrs& q_out, uint64_t* sat_partial);
hipError_t launch_int_sum(uint64_t d, const LaunchShape& ls, uint32_t n, int32_t wire,
                          const WorkerPtrs& q, int32_t* sum_out);
hipError_t launch_decode_update(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                                const int32_t* sum, const float* alpha, double eta, float* x,
                                float* gtilde_out);
hipError_t launch_update_norm(const TileMap& tm, const LaunchShape& ls, const float* x_new,
                              const float* x_old, double* norm_partial);
hipError_t launch_compress_sum(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                               const RoundSpec& rs, const WorkerPtrs& grads, const float* alpha,
                               int32_t* sum_out, uint64_t* sat_partial);
hipError_t launch_decode_update_norm(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                                     const int32_t* sum, const float* alpha, double eta, float* x,
                                     double* norm_partial);
hipError_t launch_step_fused(const TileMap& tm, const LaunchShape& ls, uint32_t n,
                             const RoundSpec& rs, const WorkerPtrs& grads, const float* alpha,
                             double eta, float* x, double* norm_partial, uint64_t* sat_partial);

// Fixed-order reduction of the per-tile norm partials into norm_sq_out[B] (skipped
// when norm_sq_out is null) and of the per-workgroup clip counts into sat_count[n]
// (skipped when sat_count is null).  tile_prefix (device, B+1 entries) gives each
// block's tile range; null means one block owning [0, num_tiles).
hipError_t launch_finalize(hipStream_t stream, const double* norm_partial,
                           const uint32_t* tile_prefix, uint32_t num_tiles, uint32_t B,
                           double* norm_sq_out, const uint64_t* sat_partial, uint32_t grid,
                           uint32_t n, uint64_t* sat_count);

// block_offsets: device array of B+1 offsets, or null when B == 1.
hipError_t launch_next_alpha(hipStream_t stream, const double* norm_sq, double* r, uint32_t B,
                             const uint64_t* block_offsets, uint64_t d, uint32_t n, double beta,
                             double eps, double eta, float* alpha_out);

}  // namespace intsgd

#endif  // INTSGD_INTERNAL_H_
