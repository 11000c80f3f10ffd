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
  const uint8_t* mask;        // B bytes, 1 = block chosen by C_step for this t
  const uint8_t* reset_mask;  // null, or B bytes: blocks C_reset chose at this t; the reset is then done in the same pass
  uint64_t ld;
  uint64_t d;
  uint32_t W;
  uint32_t block;
  float eta;
  float beta;
  uint32_t part;              // kPartAll, or one half of a launch pair (see kKernelSplit)
};

// Which column groups a fused-step launch works on.
enum StepPart : uint32_t {
  kPartAll = 0,
  kPartLocal = 1,          // only those in blocks neither compressor chose at this t
  kPartSynchronised = 2    // only those in blocks C_step (or, with a fused reset, C_reset) chose
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

// Which fused-step kernel runs (all give the same bits).
enum StepKernel {
  kKernelAuto = 0,     // by worker count and by the share of blocks that need the worker mean this iteration
  kKernelTile = 1,     // one-wavefront workgroups, one worker's row per workgroup (W <= 64)
  kKernelShared = 2,   // W-wavefront workgroups, worker sums staged in LDS (W <= 16)
  kKernelGeneral = 3,  // a lane walks all workers (any W, any block size)
  kKernelSplit = 4     // two launches: kKernelTile on the blocks neither compressor chose, then kKernelShared (W <= 16) or
                       // kKernelGeneral (more workers) on the others
};

struct Tuning {
  int kernel = kKernelAuto;
  int nontemporal = -1;     // -1 by working-set size, 0 ordinary accesses, 1 non-temporal loads and stores
  int fuse_reset = 1;       // on reset iterations do the error reset inside the fused-step kernel
  int tile_waves_per_cu = -1;    // tile kernel: most resident one-wavefront workgroups per CU; -1 by stream count, 0 no cap
  int shared_groups_per_cu = -1; // LDS-shared kernels: most resident workgroups per CU; -1 by worker count, 0 no cap
};

// Residency caps of the streaming kernels.  What the memory system rewards is a bounded number of requests in
// flight per CU; a workgroup's dynamic LDS request is the one launch parameter that bounds residency, so the
// request is chosen -- with the runtime's own occupancy calculator, for the device at hand -- as the smallest
// one under which no more than the wanted number of workgroups fit a CU.  `*_resident` is what the calculator
// reports for the chosen request (what a launch gets), 0 if it could not be queried.
struct Caps {
  uint32_t tile_lds = 0, tile_resident = 0;
  uint32_t shared_lds = 0, shared_resident = 0;         // step kernel without a fused reset
  uint32_t shared_reset_lds = 0, shared_reset_resident = 0;   // step kernel with a fused reset (twice the staging area)
  uint32_t reset_lds = 0, reset_resident = 0;           // reset kernel on its own
};
hipError_t resolve_caps(uint32_t W, bool has_e, bool has_m, bool nontemporal, const Tuning& tune, Caps* out);

// GRBS block selector (Definition 2) for the `count` iterations t0, t0 + t_stride, ...: mask[j*B + b] = 1 iff
// block b is chosen at the j-th of them.  idx (may be null, count must be 1): idx[pi^-1(b)] = b for the k chosen.
hipError_t launch_selector(uint64_t seed, uint32_t stream_id, uint64_t t0, uint64_t t_stride, uint32_t count, uint32_t B,
                           uint32_t k, uint8_t* mask, uint32_t* idx, hipStream_t s);

// The chosen block ids of a mask (16-byte aligned, holding exactly k of them) in increasing order: idx_sorted[0..k).
// counts: device scratch of kOrderedListCounts entries.
constexpr uint32_t kOrderedListCounts = 1024;
hipError_t launch_ordered_list(const uint8_t* mask, uint32_t B, uint32_t k, uint32_t* counts, uint32_t* idx_sorted,
                               hipStream_t s);

// Which kernel launch_step takes (a StepKernel other than kKernelAuto) for a launch in which `sync_share` of the
// blocks need the worker mean.  Host arithmetic only.
int choose_step_kernel(uint64_t d, uint32_t W, uint32_t block, bool vectorised, double sync_share, const Tuning& tune);

// Fused Get_p + PSync(p, C_step) + x/e update over columns [0, d) (and the error reset when p.reset_mask is set).
// `vectorised` requires block to be a multiple of 4 columns (rows need only 4-byte alignment).  `sync_share`:
// expected share of the blocks that need the worker mean in this launch.  *used (may be null) receives the kernel taken.
hipError_t launch_step(const StepParams& p, bool vectorised, bool nontemporal, const Tuning& tune, const Caps& caps,
                       double sync_share, int* used, hipStream_t s);

// Error reset on the chosen blocks (idx: the k chosen ids in increasing order; mask: the same choice as B bytes).
hipError_t launch_reset(const ResetParams& p, const uint8_t* mask, bool vectorised, bool nontemporal, const Tuning& tune,
                        const Caps& caps, hipStream_t s);

hipError_t launch_fill_zero(float* ptr, uint64_t n, hipStream_t s);
hipError_t launch_copy(void* dst, const void* src, uint64_t n_bytes, hipStream_t s);

}  // namespace cser
