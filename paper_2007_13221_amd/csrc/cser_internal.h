// Internal interface between the C ABI (cser_api.hip) and the kernels (cser_kernels.hip).
// Host-side launch wrappers only; every wrapper validates nothing (the ABI layer has done it)
// and returns the hipError_t of its launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cser {

// Everything the fused-step kernels need.  Rows are [W][ld] fp32; e and m may be null
// (implementation II of Appendix A.4 / Algorithm 2 without momentum).
struct StepParams {
  const float* g;
  float* m;
  float* x;
  float* e;
  const uint8_t* mask;  // B bytes, 1 = block chosen by C_step for this t
  const uint8_t* reset_mask;  // null, or B bytes: blocks C_reset chose at this t; the reset is then done in the same pass
  uint64_t ld;
  uint64_t d;
  uint32_t W;
  uint32_t block;
  float eta;
  float beta;
};

struct ResetParams {
  float* x;
  float* e;             // null: implementation II (average x itself)
  const uint32_t* idx;  // k chosen block ids
  uint64_t ld;
  uint64_t d;
  uint32_t W;
  uint32_t block;
  uint32_t k;
};

struct Tuning {
  int64_t wg_cap = 0;   // 0: one 4-column group per lane; > 0: at most this many workgroups
  int nontemporal = -1;  // -1 by working-set size, 0 none, 1 loads and stores, 2 loads only, 3 stores only (variant 0: zero / non-zero)
  int batch = 4;        // workers whose loads are issued together
  int threads = 64;     // workgroup size of the fused-step kernel (one wavefront: measured best)
  int variant = 1;      // 0: a lane walks all workers; row-split: 1 tiles fastest, 2 workers fastest, 3 per-XCD sweeps
  int lds_bytes = -1;   // dynamic LDS requested per workgroup and never touched (occupancy cap); -1: by stream count
  int balanced = 1;     // W a power of two <= 64: every workgroup of a tile takes 1/W of its synchronised work
  int fuse_reset = 1;   // on reset iterations do the error reset inside the fused-step kernel
  int cols_per_lane = 1;  // row-split variants: 4-column groups per lane
};

// GRBS block selector (Definition 2) for the `count` iterations t0, t0 + t_stride, ...: mask[j*B + b] = 1 iff
// block b is chosen at the j-th of them.  idx (may be null, count must be 1): idx[pi^-1(b)] = b for the k chosen.
hipError_t launch_selector(uint64_t seed, uint32_t stream_id, uint64_t t0, uint64_t t_stride, uint32_t count, uint32_t B,
                           uint32_t k, uint8_t* mask, uint32_t* idx, hipStream_t s);

// Fused Get_p + PSync(p, C_step) + x/e update over columns [0, d).  `vectorised` requires block to be a
// multiple of 4 columns (rows need only 4-byte alignment).
hipError_t launch_step(const StepParams& p, bool vectorised, const Tuning& tune, hipStream_t s);

// Error reset on the chosen blocks (idx: the k chosen ids; mask: the same choice as B bytes).
hipError_t launch_reset(const ResetParams& p, const uint8_t* mask, bool vectorised, hipStream_t s);

hipError_t launch_fill_zero(float* ptr, uint64_t n, hipStream_t s);
hipError_t launch_copy(void* dst, const void* src, uint64_t n_bytes, hipStream_t s);

}  // namespace cser
