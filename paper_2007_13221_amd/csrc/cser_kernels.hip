// HIP kernels of the CSER optimizer update for gfx950 (MI355X), and their launch wrappers.
//
//   grbs_select_kernel      the shared-seed block choice of the GRBS compressor (Definition 2, Section 3.3),
//   grbs_scatter_kernel     from the blocks' side (inverse permutation) or from the draws' side (forward)
//   cser_step_tile_kernel   Get_p + PSync(p, C_step) + the x / e updates of Algorithm 3 in one pass, and on
//                           reset iterations the error reset as well (W a power of two <= 64: the default)
//   cser_step_rows_kernel   the same for any W and other launch shapes (worker 0's workgroup walks all rows
//                           of the blocks that need the worker mean)
//   cser_step_kernel        the same, one lane per column group walking all workers (element-wise
//                           fallback for unaligned layouts; also a measured alternative)
//   cser_reset_kernel       the error-reset branch of Algorithm 3 on its own (PSync(e, C_reset), x correction)
//
// The update is a pure stream over HBM (about 6 flops per 28 bytes), so there is no matrix-core
// work here and nothing to stage in LDS.  States are worker-major rows [W][ld].  On a block that
// C_step did not choose, every worker's update is independent, so the default kernel gives each
// workgroup -- a single wavefront -- ONE worker's row over 256 columns: 4 load streams and 3 store
// streams of 128-bit accesses, 1 KiB per stream, consecutive workgroups on consecutive tiles.
// Only the chosen blocks (1 / R_step of them) need the worker mean.  In the default kernel the W
// workgroups of a tile share that work: each takes 1/W of the tile's chosen column groups for all
// workers, one worker per lane group, and the W-way sum is a fixed-order chain of wavefront
// shuffles -- every value still makes one trip, and the order is that of a sequential evaluation.
// In the general kernel a lane owns 4 columns and walks the worker axis itself (a private chain of
// adds in registers).
// What the memory system rewards, all measured: one worker per workgroup rather than all workers
// per lane, 1 KiB tiles, rows that start on 4 KiB boundaries, non-temporal accesses once the state
// exceeds the last-level cache, and no more than about 16-20 resident wavefronts per CU.
//
// Build with -ffp-contract=off: every fused multiply-add below is written out, nothing else fuses.

#include "cser_internal.h"

namespace cser {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
// The same 128-bit vector, promised to be only 4-byte aligned: gfx950 takes global_load/store_dwordx4 at any
// dword address, so rows whose start is not a multiple of 16 bytes (ld % 4 != 0, odd base addresses) still
// move 128 bits per lane; on 16-byte aligned rows the instruction is the same and nothing is lost.
typedef f4 f4_dword_aligned __attribute__((aligned(4)));

// ------------------------------------------------------------------------------------------
// V consecutive fp32 values (V = 4: one 128-bit access; V = 1: blocks that are not a multiple of 4 columns).
// ------------------------------------------------------------------------------------------
template <int V>
struct Pack {
  float v[V];
};

template <int V, bool NT>
__device__ __forceinline__ Pack<V> load_pack(const float* p) {
  Pack<V> r;
  if constexpr (V == 4) {
    f4 t;
    if constexpr (NT) t = __builtin_nontemporal_load(reinterpret_cast<const f4_dword_aligned*>(p));
    else t = *reinterpret_cast<const f4_dword_aligned*>(p);
    r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
  } else {
    if constexpr (NT) r.v[0] = __builtin_nontemporal_load(p);
    else r.v[0] = *p;
  }
  return r;
}

template <int V, bool NT>
__device__ __forceinline__ void store_pack(float* p, const Pack<V>& r) {
  if constexpr (V == 4) {
    f4 t;
    t.x = r.v[0]; t.y = r.v[1]; t.z = r.v[2]; t.w = r.v[3];
    if constexpr (NT) __builtin_nontemporal_store(t, reinterpret_cast<f4_dword_aligned*>(p));
    else *reinterpret_cast<f4_dword_aligned*>(p) = t;
  } else {
    if constexpr (NT) __builtin_nontemporal_store(r.v[0], p);
    else *p = r.v[0];
  }
}

// Get_p (Appendix A.4): m <- beta m + g, p <- eta (beta m + g); without a momentum buffer
// (beta = 0, Algorithm 2) p <- eta g.
template <int V, bool HAS_M>
__device__ __forceinline__ Pack<V> local_update(float eta, float beta, const Pack<V>& g, Pack<V>& m) {
  Pack<V> p;
#pragma unroll
  for (int c = 0; c < V; ++c) {
    if constexpr (HAS_M) {
      m.v[c] = __fmaf_rn(beta, m.v[c], g.v[c]);
      p.v[c] = eta * __fmaf_rn(beta, m.v[c], g.v[c]);
    } else {
      p.v[c] = eta * g.v[c];
    }
  }
  return p;
}

// ------------------------------------------------------------------------------------------
// Fused step.  For the V columns starting at `col`:
//   block not chosen by C_step:  C(p_i) = 0 on every worker, so the mean is 0, p'_i = r_i = p_i:
//                                x_i -= p_i, e_i -= p_i                       (28 B per element)
//   block chosen:                r_i = 0, p'_i = mean_j p_j:  x_i -= pbar, e_i untouched (20 B)
// U workers are processed per batch: all their loads are issued before any arithmetic.
// ------------------------------------------------------------------------------------------
template <int V, int U, bool NT, bool HAS_E, bool HAS_M>
__device__ __forceinline__ void step_local_batch(const StepParams& a, uint64_t col, uint32_t i0) {
  Pack<V> g[U], m[U], x[U], e[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint64_t off = static_cast<uint64_t>(i0 + u) * a.ld + col;
    g[u] = load_pack<V, NT>(a.g + off);
    if constexpr (HAS_M) m[u] = load_pack<V, NT>(a.m + off);
    x[u] = load_pack<V, NT>(a.x + off);
    if constexpr (HAS_E) e[u] = load_pack<V, NT>(a.e + off);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint64_t off = static_cast<uint64_t>(i0 + u) * a.ld + col;
    const Pack<V> p = local_update<V, HAS_M>(a.eta, a.beta, g[u], m[u]);
#pragma unroll
    for (int c = 0; c < V; ++c) {
      x[u].v[c] = x[u].v[c] - p.v[c];
      if constexpr (HAS_E) e[u].v[c] = e[u].v[c] - p.v[c];
    }
    if constexpr (HAS_M) store_pack<V, NT>(a.m + off, m[u]);
    store_pack<V, NT>(a.x + off, x[u]);
    if constexpr (HAS_E) store_pack<V, NT>(a.e + off, e[u]);
  }
}

template <int V, int U, bool NT, bool HAS_M>
__device__ __forceinline__ void step_sum_batch(const StepParams& a, uint64_t col, uint32_t i0, Pack<V>& sum) {
  Pack<V> g[U], m[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint64_t off = static_cast<uint64_t>(i0 + u) * a.ld + col;
    g[u] = load_pack<V, NT>(a.g + off);
    if constexpr (HAS_M) m[u] = load_pack<V, NT>(a.m + off);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint64_t off = static_cast<uint64_t>(i0 + u) * a.ld + col;
    const Pack<V> p = local_update<V, HAS_M>(a.eta, a.beta, g[u], m[u]);
    if constexpr (HAS_M) store_pack<V, NT>(a.m + off, m[u]);
#pragma unroll
    for (int c = 0; c < V; ++c) sum.v[c] = sum.v[c] + p.v[c];   // workers in order i = 0, 1, ...
  }
}

template <int V, int U, bool NT>
__device__ __forceinline__ void step_apply_mean_batch(const StepParams& a, uint64_t col, uint32_t i0,
                                                      const Pack<V>& pbar) {
  Pack<V> x[U];
#pragma unroll
  for (int u = 0; u < U; ++u) x[u] = load_pack<V, NT>(a.x + static_cast<uint64_t>(i0 + u) * a.ld + col);
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int c = 0; c < V; ++c) x[u].v[c] = x[u].v[c] - pbar.v[c];
    store_pack<V, NT>(a.x + static_cast<uint64_t>(i0 + u) * a.ld + col, x[u]);
  }
}

template <int V, int U, bool NT, bool HAS_E, bool HAS_M>
__device__ __forceinline__ void step_columns(const StepParams& a, uint64_t col, bool chosen) {
  if (!chosen) {
    uint32_t i = 0;
    for (; i + U <= a.W; i += U) step_local_batch<V, U, NT, HAS_E, HAS_M>(a, col, i);
    for (; i < a.W; ++i) step_local_batch<V, 1, NT, HAS_E, HAS_M>(a, col, i);
  } else {
    Pack<V> sum;
#pragma unroll
    for (int c = 0; c < V; ++c) sum.v[c] = 0.0f;
    uint32_t i = 0;
    for (; i + U <= a.W; i += U) step_sum_batch<V, U, NT, HAS_M>(a, col, i, sum);
    for (; i < a.W; ++i) step_sum_batch<V, 1, NT, HAS_M>(a, col, i, sum);
    const float n = static_cast<float>(a.W);
    Pack<V> pbar;
#pragma unroll
    for (int c = 0; c < V; ++c) pbar.v[c] = sum.v[c] / n;
    i = 0;
    for (; i + U <= a.W; i += U) step_apply_mean_batch<V, U, NT>(a, col, i, pbar);
    for (; i < a.W; ++i) step_apply_mean_batch<V, 1, NT>(a, col, i, pbar);
  }
}

// Chosen block, W <= 8: the same arithmetic as the chosen branch of step_columns, but g, m and x of all
// workers are requested in one go and held in registers, so the lane waits for memory once
// instead of four times (loads of absent workers i >= W are skipped, their slots unused).
template <int V, bool NT, bool HAS_M>
__device__ __forceinline__ void step_chosen_up_to_8(const StepParams& a, uint64_t col) {
  Pack<V> g[8], m[8], x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (static_cast<uint32_t>(i) < a.W) {
      const uint64_t off = static_cast<uint64_t>(i) * a.ld + col;
      g[i] = load_pack<V, NT>(a.g + off);
      if constexpr (HAS_M) m[i] = load_pack<V, NT>(a.m + off);
      x[i] = load_pack<V, NT>(a.x + off);
    }
  }
  Pack<V> sum;
#pragma unroll
  for (int c = 0; c < V; ++c) sum.v[c] = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (static_cast<uint32_t>(i) < a.W) {
      const Pack<V> p = local_update<V, HAS_M>(a.eta, a.beta, g[i], m[i]);
      if constexpr (HAS_M) store_pack<V, NT>(a.m + static_cast<uint64_t>(i) * a.ld + col, m[i]);
#pragma unroll
      for (int c = 0; c < V; ++c) sum.v[c] = sum.v[c] + p.v[c];   // workers in order i = 0, 1, ...
    }
  }
  const float n = static_cast<float>(a.W);
  Pack<V> pbar;
#pragma unroll
  for (int c = 0; c < V; ++c) pbar.v[c] = sum.v[c] / n;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (static_cast<uint32_t>(i) < a.W) {
#pragma unroll
      for (int c = 0; c < V; ++c) x[i].v[c] = x[i].v[c] - pbar.v[c];
      store_pack<V, NT>(a.x + static_cast<uint64_t>(i) * a.ld + col, x[i]);
    }
  }
}

// Reset iterations (t mod H = 0) with the reset fused into the step: the V columns at `col` belong
// to a block C_reset chose, so after the step's own update the error reset follows at once,
//   ebar = (e'_0 + ... + e'_{W-1}) / W ;  x_i <- (x'_i - e'_i) + ebar ;  e_i <- +0
// (implementation II: x_i <- (x'_0 + ... + x'_{W-1}) / W), where x', e' are the values after the
// step.  Every operation and its order are those of running the step kernel and then the reset
// kernel; x and e just travel through registers instead of memory.  A worker's update p_i is
// recomputed from g_i and the old m_i in each pass (m is stored only in the last), so no pass reads
// what an earlier pass wrote.  Plain (temporal) accesses: the re-reads are meant to hit in L2.
template <int V, bool HAS_E, bool HAS_M>
__device__ __forceinline__ void step_and_reset_columns(const StepParams& a, uint64_t col, bool step_chosen) {
  const float n = static_cast<float>(a.W);
  Pack<V> pbar, sum, mean, zero;
#pragma unroll
  for (int c = 0; c < V; ++c) {
    pbar.v[c] = 0.0f;
    sum.v[c] = 0.0f;
    zero.v[c] = 0.0f;
  }
  if (step_chosen) {   // pbar = mean_i p_i
    Pack<V> psum = zero;
    for (uint32_t i = 0; i < a.W; ++i) {
      const uint64_t off = static_cast<uint64_t>(i) * a.ld + col;
      const Pack<V> g = load_pack<V, false>(a.g + off);
      Pack<V> m = zero;
      if constexpr (HAS_M) m = load_pack<V, false>(a.m + off);
      const Pack<V> p = local_update<V, HAS_M>(a.eta, a.beta, g, m);
#pragma unroll
      for (int c = 0; c < V; ++c) psum.v[c] = psum.v[c] + p.v[c];
    }
#pragma unroll
    for (int c = 0; c < V; ++c) pbar.v[c] = psum.v[c] / n;
  }
  // worker sum of what the reset averages: e after the step (implementation I) or x after the step (II)
  for (uint32_t i = 0; i < a.W; ++i) {
    const uint64_t off = static_cast<uint64_t>(i) * a.ld + col;
    Pack<V> v = load_pack<V, false>((HAS_E ? a.e : a.x) + off);
    if (!step_chosen) {
      const Pack<V> g = load_pack<V, false>(a.g + off);
      Pack<V> m = zero;
      if constexpr (HAS_M) m = load_pack<V, false>(a.m + off);
      const Pack<V> p = local_update<V, HAS_M>(a.eta, a.beta, g, m);
#pragma unroll
      for (int c = 0; c < V; ++c) v.v[c] = v.v[c] - p.v[c];        // e - r  or  x - p'
    } else if constexpr (!HAS_E) {
#pragma unroll
      for (int c = 0; c < V; ++c) v.v[c] = v.v[c] - pbar.v[c];     // x - pbar (e is untouched on chosen blocks)
    }
#pragma unroll
    for (int c = 0; c < V; ++c) sum.v[c] = sum.v[c] + v.v[c];
  }
#pragma unroll
  for (int c = 0; c < V; ++c) mean.v[c] = sum.v[c] / n;
  // apply
  for (uint32_t i = 0; i < a.W; ++i) {
    const uint64_t off = static_cast<uint64_t>(i) * a.ld + col;
    const Pack<V> g = load_pack<V, false>(a.g + off);
    Pack<V> m = zero;
    if constexpr (HAS_M) m = load_pack<V, false>(a.m + off);
    const Pack<V> p = local_update<V, HAS_M>(a.eta, a.beta, g, m);
    if constexpr (HAS_M) store_pack<V, false>(a.m + off, m);
    if constexpr (HAS_E) {
      Pack<V> x = load_pack<V, false>(a.x + off);
      Pack<V> e = load_pack<V, false>(a.e + off);
#pragma unroll
      for (int c = 0; c < V; ++c) {
        x.v[c] = x.v[c] - (step_chosen ? pbar.v[c] : p.v[c]);
        if (!step_chosen) e.v[c] = e.v[c] - p.v[c];
        x.v[c] = (x.v[c] - e.v[c]) + mean.v[c];
      }
      store_pack<V, false>(a.x + off, x);
      store_pack<V, false>(a.e + off, zero);
    } else {
      store_pack<V, false>(a.x + off, mean);
    }
  }
}

// Columns [col_begin, col_end) in groups of V; group q covers col_begin + q*V ...  `groups` is
// the number of whole groups.  groups_per_block = block / V (vector path: block % 4 == 0 and
// col_begin % block == 0, so a group never straddles two blocks).
template <int V, int U, bool NT, bool HAS_E, bool HAS_M>
__global__ __launch_bounds__(1024) void cser_step_kernel(StepParams a, uint64_t col_begin, uint32_t groups) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  for (uint64_t q = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; q < groups; q += stride) {
    const uint64_t col = col_begin + q * V;
    uint32_t b;
    if constexpr (V == 4) b = static_cast<uint32_t>(q) / (a.block / 4u);   // vector path starts at column 0
    else b = static_cast<uint32_t>(col / a.block);
    const bool step_chosen = a.mask[b] != 0;
    if (a.reset_mask != nullptr && a.reset_mask[b] != 0) step_and_reset_columns<V, HAS_E, HAS_M>(a, col, step_chosen);
    else step_columns<V, U, NT, HAS_E, HAS_M>(a, col, step_chosen);
  }
}

// Row-split variant of the vector path.  A workgroup owns one worker's row over a tile of
// C * blockDim.x column groups (each lane takes C groups spaced blockDim.x apart, so every access
// stays coalesced): unchosen blocks need nothing from the other workers.  Chosen blocks need the
// worker mean (and so do the blocks C_reset chose, on a reset iteration with the reset fused in);
// the workgroup of worker 0 walks all rows for those.
// `order` maps the workgroup id to its (worker, tile) pair:
//   0  tiles fastest: consecutive workgroups sweep one worker's row, then the next worker's
//   1  workers fastest: consecutive workgroups take the same tile of every worker
//   2  as 0, but the ids are first regrouped so that each of the 8 XCDs (ids are dealt to them
//      round-robin) sweeps one contiguous eighth of the (worker, tile) sequence
// NTMODE: bit 0 = non-temporal loads, bit 1 = non-temporal stores.
template <int C, int NTMODE, bool HAS_E, bool HAS_M>
__global__ __launch_bounds__(1024) void cser_step_rows_kernel(StepParams a, uint32_t groups, uint32_t tiles,
                                                               uint32_t order) {
  constexpr bool NTL = (NTMODE & 1) != 0, NTS = (NTMODE & 2) != 0;
  uint32_t tile, i;
  if (order == 1) {
    tile = blockIdx.x / a.W;
    i = blockIdx.x - tile * a.W;
  } else {
    uint32_t linear = blockIdx.x;
    if (order == 2) {
      const uint32_t per_xcd = gridDim.x / 8u;   // the launcher rounds the grid up to a multiple of 8
      linear = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
      if (linear >= tiles * a.W) return;
    }
    i = linear / tiles;
    tile = linear - i * tiles;
  }
  const uint64_t row = static_cast<uint64_t>(i) * a.ld;
  const uint32_t groups_per_block = a.block / 4u;
  uint32_t q[C];
  bool local[C], chosen[C], reset_chosen[C];
  Pack<4> g[C], m[C], x[C], e[C];
#pragma unroll
  for (int c = 0; c < C; ++c) {
    const uint64_t q64 = (static_cast<uint64_t>(tile) * C + c) * blockDim.x + threadIdx.x;
    const bool live = q64 < groups;
    q[c] = live ? static_cast<uint32_t>(q64) : 0u;
    const uint32_t b = q[c] / groups_per_block;
    chosen[c] = live && a.mask[b] != 0;
    reset_chosen[c] = live && a.reset_mask != nullptr && a.reset_mask[b] != 0;
    local[c] = live && !chosen[c] && !reset_chosen[c];
    if (local[c]) {
      const uint64_t off = row + static_cast<uint64_t>(q[c]) * 4;
      g[c] = load_pack<4, NTL>(a.g + off);
      if constexpr (HAS_M) m[c] = load_pack<4, NTL>(a.m + off);
      x[c] = load_pack<4, NTL>(a.x + off);
      if constexpr (HAS_E) e[c] = load_pack<4, NTL>(a.e + off);
    }
  }
#pragma unroll
  for (int c = 0; c < C; ++c) {
    if (local[c]) {
      const uint64_t off = row + static_cast<uint64_t>(q[c]) * 4;
      const Pack<4> p = local_update<4, HAS_M>(a.eta, a.beta, g[c], m[c]);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        x[c].v[k] = x[c].v[k] - p.v[k];
        if constexpr (HAS_E) e[c].v[k] = e[c].v[k] - p.v[k];
      }
      if constexpr (HAS_M) store_pack<4, NTS>(a.m + off, m[c]);
      store_pack<4, NTS>(a.x + off, x[c]);
      if constexpr (HAS_E) store_pack<4, NTS>(a.e + off, e[c]);
    }
  }
  if (i == 0) {
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const uint64_t col = static_cast<uint64_t>(q[c]) * 4;
      if (reset_chosen[c]) step_and_reset_columns<4, HAS_E, HAS_M>(a, col, chosen[c]);
      else if (chosen[c]) {
        if (a.W <= 8) step_chosen_up_to_8<4, NTL && NTS, HAS_M>(a, col);
        else step_columns<4, 4, NTL && NTS, HAS_E, HAS_M>(a, col, true);
      }
    }
  }
}

// Ordered worker sum inside one wavefront.  Lanes are laid out as (worker j, group k) = (lane / G,
// lane % G); every lane fetches the W values of its group k with wavefront shuffles and adds them in
// the order j = 0, 1, ..., W-1 -- the order of a sequential evaluation -- so all W lanes of a group
// end up with the same bits.  Must be called with all 64 lanes active.
template <int V>
__device__ __forceinline__ Pack<V> worker_sum_in_wave(const Pack<V>& v, uint32_t W, uint32_t G, uint32_t k) {
  Pack<V> sum;
#pragma unroll
  for (int c = 0; c < V; ++c) sum.v[c] = 0.0f;
  for (uint32_t j = 0; j < W; ++j) {
    const int src = static_cast<int>(j * G + k);
#pragma unroll
    for (int c = 0; c < V; ++c) sum.v[c] = sum.v[c] + __shfl(v.v[c], src, 64);
  }
  return sum;
}

// Balanced row-split kernel for W a power of two up to 64; one wavefront per workgroup, which owns
// the pair (worker i, tile of 64 column groups = 256 columns) and plays two roles:
//   A  lane l takes column group l of the tile in worker i's row, if its block was chosen by neither
//      compressor: the purely local update, as in cser_step_rows_kernel;
//   B  the tile's column groups are cut into W slices of G = 64 / W groups; this workgroup takes
//      slice i for ALL workers: lane (j, k) holds worker j's values of group i*G + k.  For groups
//      whose block C_step chose, pbar is the in-wavefront ordered sum over j divided by W; for groups
//      C_reset chose on a reset iteration the error reset follows at once, from registers:
//      ebar = ordered sum of the post-step e_j / W, x_j <- (x_j - e_j) + ebar, e_j <- +0
//      (implementation II: x_j <- ordered sum of the post-step x_j / W).
// Every workgroup of a tile thus does 1/W of the tile's synchronised work, whatever share of the
// blocks is chosen, and each value is read and written exactly once.  The arithmetic and its order
// are those of the other kernels.
template <int NTMODE, bool HAS_E, bool HAS_M>
__global__ __launch_bounds__(64) void cser_step_tile_kernel(StepParams a, uint32_t groups, uint32_t tiles,
                                                             uint32_t order, uint32_t log2_w) {
  constexpr bool NTL = (NTMODE & 1) != 0, NTS = (NTMODE & 2) != 0;
  uint32_t tile, i;
  if (order == 1) {
    tile = blockIdx.x >> log2_w;
    i = blockIdx.x & (a.W - 1u);
  } else {
    uint32_t linear = blockIdx.x;
    if (order == 2) {
      const uint32_t per_xcd = gridDim.x / 8u;   // the launcher rounds the grid up to a multiple of 8
      linear = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
      if (linear >= tiles * a.W) return;         // uniform over the workgroup
    }
    i = linear / tiles;
    tile = linear - i * tiles;
  }
  const uint32_t lane = threadIdx.x;
  const uint32_t groups_per_block = a.block / 4u;
  const uint32_t G = 64u >> log2_w;              // column groups per slice
  const uint32_t j = lane / G, k = lane - j * G; // role B: worker j, group k of slice i
  const uint64_t tile_first = static_cast<uint64_t>(tile) * 64u;

  // role A
  const uint64_t qa = tile_first + lane;
  const bool live_a = qa < groups;
  const uint32_t ba = static_cast<uint32_t>(live_a ? qa : 0u) / groups_per_block;
  const bool local_a = live_a && a.mask[ba] == 0 && (a.reset_mask == nullptr || a.reset_mask[ba] == 0);
  // role B
  const uint64_t qb = tile_first + static_cast<uint64_t>(i) * G + k;
  const bool live_b = qb < groups;
  const uint32_t bb = static_cast<uint32_t>(live_b ? qb : 0u) / groups_per_block;
  const bool step_b = live_b && a.mask[bb] != 0;
  const bool reset_b = live_b && a.reset_mask != nullptr && a.reset_mask[bb] != 0;
  const bool sync_b = step_b || reset_b;

  const uint64_t off_a = static_cast<uint64_t>(i) * a.ld + qa * 4u;
  const uint64_t off_b = static_cast<uint64_t>(j) * a.ld + qb * 4u;
  Pack<4> ga, ma, xa, ea, gb, mb, xb, eb;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    gb.v[c] = 0.0f; mb.v[c] = 0.0f; xb.v[c] = 0.0f; eb.v[c] = 0.0f;
  }
  if (local_a) {
    ga = load_pack<4, NTL>(a.g + off_a);
    if constexpr (HAS_M) ma = load_pack<4, NTL>(a.m + off_a);
    xa = load_pack<4, NTL>(a.x + off_a);
    if constexpr (HAS_E) ea = load_pack<4, NTL>(a.e + off_a);
  }
  if (sync_b) {
    gb = load_pack<4, NTL>(a.g + off_b);
    if constexpr (HAS_M) mb = load_pack<4, NTL>(a.m + off_b);
    xb = load_pack<4, NTL>(a.x + off_b);
    if constexpr (HAS_E) {
      if (reset_b) eb = load_pack<4, NTL>(a.e + off_b);   // e is untouched by the step on a block C_step chose
    }
  }
  if (local_a) {
    const Pack<4> p = local_update<4, HAS_M>(a.eta, a.beta, ga, ma);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      xa.v[c] = xa.v[c] - p.v[c];
      if constexpr (HAS_E) ea.v[c] = ea.v[c] - p.v[c];
    }
    if constexpr (HAS_M) store_pack<4, NTS>(a.m + off_a, ma);
    store_pack<4, NTS>(a.x + off_a, xa);
    if constexpr (HAS_E) store_pack<4, NTS>(a.e + off_a, ea);
  }
  if (__any(sync_b)) {   // wavefront-uniform: all 64 lanes take part in the shuffles below
    Pack<4> p;
#pragma unroll
    for (int c = 0; c < 4; ++c) p.v[c] = 0.0f;
    if (sync_b) {
      p = local_update<4, HAS_M>(a.eta, a.beta, gb, mb);
      if constexpr (HAS_M) store_pack<4, NTS>(a.m + off_b, mb);
    }
    const float n = static_cast<float>(a.W);
    if (__any(step_b)) {
      const Pack<4> psum = worker_sum_in_wave<4>(p, a.W, G, k);
      if (step_b) {
#pragma unroll
        for (int c = 0; c < 4; ++c) p.v[c] = psum.v[c] / n;   // p' = pbar, r = 0
      }
    }
    if (sync_b) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        xb.v[c] = xb.v[c] - p.v[c];
        if constexpr (HAS_E) {
          if (!step_b) eb.v[c] = eb.v[c] - p.v[c];            // r = p off the blocks C_step chose
        }
      }
    }
    if (__any(reset_b)) {
      Pack<4> v;
#pragma unroll
      for (int c = 0; c < 4; ++c) v.v[c] = reset_b ? (HAS_E ? eb.v[c] : xb.v[c]) : 0.0f;
      const Pack<4> vsum = worker_sum_in_wave<4>(v, a.W, G, k);
      if (reset_b) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float mean = vsum.v[c] / n;
          if constexpr (HAS_E) {
            xb.v[c] = (xb.v[c] - eb.v[c]) + mean;
            eb.v[c] = 0.0f;
          } else {
            xb.v[c] = mean;
          }
        }
      }
    }
    if (sync_b) {
      store_pack<4, NTS>(a.x + off_b, xb);
      if constexpr (HAS_E) {
        if (reset_b) store_pack<4, NTS>(a.e + off_b, eb);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Error reset (Algorithm 3, t mod H = 0) on the V columns at `col` of a chosen block:
//   ebar = (e_0 + e_1 + ... + e_{W-1}) / W ;  x_i <- (x_i - e_i) + ebar ;  e_i <- +0
// Implementation II (no e): x_i <- (x_0 + ... + x_{W-1}) / W.
// The second pass re-reads e_i; the lines were just fetched by this lane, so they come from L2.
// ------------------------------------------------------------------------------------------
template <int V, bool HAS_E>
__device__ __forceinline__ void reset_columns(const ResetParams& a, uint64_t col) {
  float* src = HAS_E ? a.e : a.x;
  Pack<V> sum;
#pragma unroll
  for (int c = 0; c < V; ++c) sum.v[c] = 0.0f;
  for (uint32_t i = 0; i < a.W; ++i) {
    const Pack<V> v = load_pack<V, false>(src + static_cast<uint64_t>(i) * a.ld + col);
#pragma unroll
    for (int c = 0; c < V; ++c) sum.v[c] = sum.v[c] + v.v[c];
  }
  const float n = static_cast<float>(a.W);
  Pack<V> mean, zero;
#pragma unroll
  for (int c = 0; c < V; ++c) {
    mean.v[c] = sum.v[c] / n;
    zero.v[c] = 0.0f;
  }
  for (uint32_t i = 0; i < a.W; ++i) {
    const uint64_t off = static_cast<uint64_t>(i) * a.ld + col;
    if constexpr (HAS_E) {
      const Pack<V> e = load_pack<V, false>(a.e + off);
      Pack<V> x = load_pack<V, false>(a.x + off);
#pragma unroll
      for (int c = 0; c < V; ++c) x.v[c] = (x.v[c] - e.v[c]) + mean.v[c];
      store_pack<V, false>(a.x + off, x);
      store_pack<V, false>(a.e + off, zero);
    } else {
      store_pack<V, false>(a.x + off, mean);
    }
  }
}

// Vector path: one lane per 4-column group of a chosen block; the block list comes from idx.
template <bool HAS_E>
__global__ __launch_bounds__(256) void cser_reset_kernel(ResetParams a, uint32_t groups_per_block,
                                                          uint64_t total_groups) {
  const uint64_t q = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (q >= total_groups) return;
  const uint32_t j = static_cast<uint32_t>(q / groups_per_block);
  const uint32_t within = static_cast<uint32_t>(q - static_cast<uint64_t>(j) * groups_per_block);
  const uint64_t col = static_cast<uint64_t>(a.idx[j]) * a.block + static_cast<uint64_t>(within) * 4;
  if (col + 4 > a.d) return;   // ragged last block; a trailing partial group goes to the scalar kernel
  reset_columns<4, HAS_E>(a, col);
}

// Element-wise path over columns [col_begin, col_end): uses the mask, any alignment.
template <bool HAS_E>
__global__ __launch_bounds__(256) void cser_reset_scalar_kernel(ResetParams a, const uint8_t* mask,
                                                                 uint64_t col_begin, uint64_t col_end) {
  const uint64_t col = col_begin + static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (col >= col_end) return;
  if (mask[col / a.block] == 0) return;
  reset_columns<1, HAS_E>(a, col);
}

// ------------------------------------------------------------------------------------------
// Block selector.  All workers must pick the same k of the B blocks from a shared seed
// (Definition 2).  The choice is {pi(0), ..., pi(k-1)} for a keyed permutation pi of [0, B):
// block b is chosen iff pi^-1(b) < k, which every block can decide for itself -- no sort, no
// atomics, one thread per block.
//
// pi: 8-round balanced Feistel network on 2h bits (2^(2h) >= B), round function = low h bits of
// word 0 of Philox-4x32-10 (Salmon et al., SC'11) keyed by the seed with counter
// (half, stream*65536 + round, t_lo, t_hi); values >= B are walked through the network again
// (cycle walking).  This kernel evaluates the inverse.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t philox_first_word(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                      uint32_t k0, uint32_t k1) {
  constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
  constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hiA = __umulhi(kMulA, c0), loA = kMulA * c0;
    const uint32_t hiB = __umulhi(kMulB, c2), loB = kMulB * c2;
    c0 = hiB ^ c1 ^ k0;
    c1 = loB;
    c2 = hiA ^ c3 ^ k1;
    c3 = loA;
    k0 += kWeylA;
    k1 += kWeylB;
  }
  return c0;
}

// blockIdx.y selects the iteration t0 + blockIdx.y * t_stride (the choice is a pure function of t, so several
// iterations can be drawn ahead in one launch); its mask goes to mask + blockIdx.y * B.  idx may be
// null; when given it is only meaningful for a launch with gridDim.y == 1.
__global__ __launch_bounds__(256) void grbs_select_kernel(uint32_t seed_lo, uint32_t seed_hi, uint32_t stream_id,
                                                           uint64_t t0, uint64_t t_stride, uint32_t B, uint32_t k,
                                                           uint32_t half_bits, uint8_t* mask, uint32_t* idx) {
  const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const uint64_t t = t0 + blockIdx.y * t_stride;
  const uint32_t t_lo = static_cast<uint32_t>(t), t_hi = static_cast<uint32_t>(t >> 32);
  mask += static_cast<uint64_t>(blockIdx.y) * B;
  const uint32_t half_mask = (1u << half_bits) - 1u;
  // The network is a bijection of the 2^(2h) values, so the walk from b returns to b after at most
  // 2^(2h) applications and passes a value < B no later than that: the bound below is never the
  // reason the loop ends, it only makes termination independent of that argument.
  const uint64_t domain = 1ull << (2 * half_bits);
  uint32_t v = b;
  for (uint64_t walk = 0; walk < domain; ++walk) {
    uint32_t hi = (v >> half_bits) & half_mask;
    uint32_t lo = v & half_mask;
    // undo rounds 7..0 of (L, R) -> (R, L ^ F(round, R)):  given (hi, lo) = (R, L ^ F), recover (L, R)
    for (int round = 7; round >= 0; --round) {
      const uint32_t f = philox_first_word(hi, stream_id * 65536u + static_cast<uint32_t>(round), t_lo, t_hi,
                                           seed_lo, seed_hi) & half_mask;
      const uint32_t prev_left = lo ^ f;
      lo = hi;
      hi = prev_left;
    }
    v = (hi << half_bits) | lo;
    if (v < B) break;
  }
  const bool chosen = v < k;
  mask[b] = chosen ? 1 : 0;
  if (chosen && idx != nullptr) idx[v] = b;
}

// The same choice from the other side: a thread evaluates pi(j) with the forward network and writes
// `value` into that block's byte of a mask that was filled with the opposite value beforehand.
// Draws j in [0, k) with value 1 on a zeroed mask mark the chosen blocks (k evaluations); draws j in
// [k, B) with value 0 on a mask of ones clear the unchosen ones (B - k evaluations).  Whichever is
// smaller costs less than the B evaluations of grbs_select_kernel; all forms give the same mask
// because pi is a bijection.  idx (may be null) is only meaningful for the first form.
__global__ __launch_bounds__(256) void grbs_scatter_kernel(uint32_t seed_lo, uint32_t seed_hi, uint32_t stream_id,
                                                            uint64_t t0, uint64_t t_stride, uint32_t B, uint32_t j_begin,
                                                            uint32_t j_end, uint8_t value, uint32_t half_bits,
                                                            uint8_t* mask, uint32_t* idx) {
  const uint32_t j = j_begin + blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= j_end) return;
  const uint64_t t = t0 + blockIdx.y * t_stride;
  const uint32_t t_lo = static_cast<uint32_t>(t), t_hi = static_cast<uint32_t>(t >> 32);
  mask += static_cast<uint64_t>(blockIdx.y) * B;
  const uint32_t half_mask = (1u << half_bits) - 1u;
  const uint64_t domain = 1ull << (2 * half_bits);   // bound of the cycle walk, as in grbs_select_kernel
  uint32_t v = j;
  for (uint64_t walk = 0; walk < domain; ++walk) {
    uint32_t left = (v >> half_bits) & half_mask;
    uint32_t right = v & half_mask;
    for (uint32_t round = 0; round < 8; ++round) {   // (L, R) -> (R, L ^ F(round, R))
      const uint32_t f = philox_first_word(right, stream_id * 65536u + round, t_lo, t_hi, seed_lo, seed_hi) & half_mask;
      const uint32_t next_right = left ^ f;
      left = right;
      right = next_right;
    }
    v = (left << half_bits) | right;
    if (v < B) break;
  }
  if (v < B) {   // always true (see the bound above); keeps a write in range whatever happens
    mask[v] = value;
    if (idx != nullptr) idx[j] = v;
  }
}

__global__ __launch_bounds__(256) void fill_bytes_kernel(uint8_t* p, uint64_t n, uint8_t value) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  const uint64_t n4 = n / 4;   // p comes from hipMalloc: 4-byte aligned
  uint32_t* p4 = reinterpret_cast<uint32_t*>(p);
  const uint32_t word = value * 0x01010101u;
  for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n4; i += stride) p4[i] = word;
  if (blockIdx.x == 0 && threadIdx.x < n - n4 * 4) p[n4 * 4 + threadIdx.x] = value;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* p, uint64_t n) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.0f;
}

__global__ __launch_bounds__(256) void copy_kernel(f4* __restrict__ dst, const f4* __restrict__ src, uint64_t n16) {
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// ---------------------------------------------------------------- launch helpers
uint32_t half_bits_for(uint32_t B) {
  uint32_t bits = 0;
  while ((1ull << bits) < B) ++bits;
  if (bits < 2) bits = 2;
  return (bits + 1) / 2;
}

template <int V, int U, bool NT>
hipError_t launch_step_flags(const StepParams& p, uint64_t col_begin, uint32_t groups, uint32_t grid, uint32_t threads,
                             hipStream_t s) {
  const bool has_e = p.e != nullptr, has_m = p.m != nullptr;
  if (has_e && has_m) hipLaunchKernelGGL((cser_step_kernel<V, U, NT, true, true>), dim3(grid), dim3(threads), 0, s, p, col_begin, groups);
  else if (has_e && !has_m) hipLaunchKernelGGL((cser_step_kernel<V, U, NT, true, false>), dim3(grid), dim3(threads), 0, s, p, col_begin, groups);
  else if (!has_e && has_m) hipLaunchKernelGGL((cser_step_kernel<V, U, NT, false, true>), dim3(grid), dim3(threads), 0, s, p, col_begin, groups);
  else hipLaunchKernelGGL((cser_step_kernel<V, U, NT, false, false>), dim3(grid), dim3(threads), 0, s, p, col_begin, groups);
  return hipGetLastError();
}

template <int V, bool NT>
hipError_t launch_step_batch(const StepParams& p, uint64_t col_begin, uint32_t groups, uint32_t grid, uint32_t threads,
                             int batch, hipStream_t s) {
  switch (batch) {
    case 1: return launch_step_flags<V, 1, NT>(p, col_begin, groups, grid, threads, s);
    case 2: return launch_step_flags<V, 2, NT>(p, col_begin, groups, grid, threads, s);
    case 8: return launch_step_flags<V, 8, NT>(p, col_begin, groups, grid, threads, s);
    default: return launch_step_flags<V, 4, NT>(p, col_begin, groups, grid, threads, s);
  }
}

template <int V>
hipError_t launch_step_range(const StepParams& p, uint64_t col_begin, uint64_t col_end, const Tuning& tune,
                             hipStream_t s) {
  if (col_end <= col_begin) return hipSuccess;
  const uint64_t groups64 = (col_end - col_begin) / V;
  if (groups64 == 0) return hipSuccess;
  const uint32_t groups = static_cast<uint32_t>(groups64);
  const uint32_t threads = static_cast<uint32_t>(tune.threads);
  uint64_t grid = (groups64 + threads - 1) / threads;
  if (tune.wg_cap > 0 && grid > static_cast<uint64_t>(tune.wg_cap)) grid = static_cast<uint64_t>(tune.wg_cap);
  if (tune.nontemporal) return launch_step_batch<V, true>(p, col_begin, groups, static_cast<uint32_t>(grid), threads, tune.batch, s);
  return launch_step_batch<V, false>(p, col_begin, groups, static_cast<uint32_t>(grid), threads, tune.batch, s);
}

// Occupancy cap of the row-split kernels: bytes of dynamic LDS requested per one-wavefront workgroup and
// never touched.  What the memory system likes is a bounded number of requests in flight per CU, so the
// cap follows the number of load streams per wavefront: 4 streams (g, m, x, e) -> 8 KiB = 20 wavefronts
// per CU, 3 streams -> 7 KiB = 22, 2 streams (x only) -> no cap (measured: each is the best or within
// 0.5 % of the best of a sweep, and 4-19 % better than the wrong one).
uint32_t resolve_lds(const StepParams& p, const Tuning& tune) {
  if (tune.lds_bytes >= 0) return static_cast<uint32_t>(tune.lds_bytes);
  const int streams = 2 + (p.e != nullptr ? 1 : 0) + (p.m != nullptr ? 1 : 0);
  return streams >= 4 ? 8192u : (streams == 3 ? 7168u : 0u);
}

int resolve_nontemporal(const StepParams& p, const Tuning& tune) {
  int mode = tune.nontemporal;
  if (mode < 0) {
    // automatic: a working set that fits the 256 MiB last-level cache is better served by ordinary accesses
    // (x, e, m come back next iteration; measured +7 % at 110-250 MB), a larger one by non-temporal ones (+10 %)
    const uint64_t arrays = 2u + (p.e != nullptr ? 1u : 0u) + (p.m != nullptr ? 1u : 0u);
    mode = static_cast<uint64_t>(p.W) * p.ld * 4u * arrays <= (256ull << 20) ? 0 : 1;
  }
  return mode;
}

template <int C, int NTMODE>
hipError_t launch_rows_flags(const StepParams& p, uint32_t groups, uint32_t tiles, uint32_t grid_size, uint32_t threads,
                             uint32_t order, uint32_t lds, hipStream_t s) {
  const bool has_e = p.e != nullptr, has_m = p.m != nullptr;
  const dim3 grid(grid_size), block(threads);
  if (has_e && has_m) hipLaunchKernelGGL((cser_step_rows_kernel<C, NTMODE, true, true>), grid, block, lds, s, p, groups, tiles, order);
  else if (has_e && !has_m) hipLaunchKernelGGL((cser_step_rows_kernel<C, NTMODE, true, false>), grid, block, lds, s, p, groups, tiles, order);
  else if (!has_e && has_m) hipLaunchKernelGGL((cser_step_rows_kernel<C, NTMODE, false, true>), grid, block, lds, s, p, groups, tiles, order);
  else hipLaunchKernelGGL((cser_step_rows_kernel<C, NTMODE, false, false>), grid, block, lds, s, p, groups, tiles, order);
  return hipGetLastError();
}

template <int C>
hipError_t launch_rows_c(const StepParams& p, uint32_t groups, const Tuning& tune, hipStream_t s) {
  const uint32_t threads = static_cast<uint32_t>(tune.threads);
  const uint64_t per_tile = static_cast<uint64_t>(threads) * C;
  const uint64_t tiles64 = (groups + per_tile - 1) / per_tile;
  const uint32_t order = tune.variant == 2 ? 1u : (tune.variant == 3 ? 2u : 0u);
  uint64_t grid64 = tiles64 * p.W;
  if (order == 2) grid64 = (grid64 + 7) / 8 * 8;
  if (grid64 > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
  const uint32_t tiles = static_cast<uint32_t>(tiles64), grid = static_cast<uint32_t>(grid64);
  const uint32_t lds = resolve_lds(p, tune);
  switch (resolve_nontemporal(p, tune)) {
    case 0: return launch_rows_flags<C, 0>(p, groups, tiles, grid, threads, order, lds, s);
    case 2: return launch_rows_flags<C, 1>(p, groups, tiles, grid, threads, order, lds, s);
    case 3: return launch_rows_flags<C, 2>(p, groups, tiles, grid, threads, order, lds, s);
    default: return launch_rows_flags<C, 3>(p, groups, tiles, grid, threads, order, lds, s);
  }
}

template <int NTMODE>
hipError_t launch_tile_flags(const StepParams& p, uint32_t groups, uint32_t tiles, uint32_t grid_size, uint32_t order,
                             uint32_t log2_w, uint32_t lds, hipStream_t s) {
  const bool has_e = p.e != nullptr, has_m = p.m != nullptr;
  const dim3 grid(grid_size), block(64);
  if (has_e && has_m) hipLaunchKernelGGL((cser_step_tile_kernel<NTMODE, true, true>), grid, block, lds, s, p, groups, tiles, order, log2_w);
  else if (has_e && !has_m) hipLaunchKernelGGL((cser_step_tile_kernel<NTMODE, true, false>), grid, block, lds, s, p, groups, tiles, order, log2_w);
  else if (!has_e && has_m) hipLaunchKernelGGL((cser_step_tile_kernel<NTMODE, false, true>), grid, block, lds, s, p, groups, tiles, order, log2_w);
  else hipLaunchKernelGGL((cser_step_tile_kernel<NTMODE, false, false>), grid, block, lds, s, p, groups, tiles, order, log2_w);
  return hipGetLastError();
}

// The balanced kernel: W a power of two <= 64, one-wavefront workgroups, one column group per lane.
hipError_t launch_tile(const StepParams& p, uint32_t groups, const Tuning& tune, hipStream_t s) {
  uint32_t log2_w = 0;
  while ((1u << log2_w) < p.W) ++log2_w;
  const uint64_t tiles64 = (static_cast<uint64_t>(groups) + 63) / 64;
  const uint32_t order = tune.variant == 2 ? 1u : (tune.variant == 3 ? 2u : 0u);
  uint64_t grid64 = tiles64 * p.W;
  if (order == 2) grid64 = (grid64 + 7) / 8 * 8;
  if (grid64 > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
  const uint32_t tiles = static_cast<uint32_t>(tiles64), grid = static_cast<uint32_t>(grid64);
  const uint32_t lds = resolve_lds(p, tune);
  switch (resolve_nontemporal(p, tune)) {
    case 0: return launch_tile_flags<0>(p, groups, tiles, grid, order, log2_w, lds, s);
    case 2: return launch_tile_flags<1>(p, groups, tiles, grid, order, log2_w, lds, s);
    case 3: return launch_tile_flags<2>(p, groups, tiles, grid, order, log2_w, lds, s);
    default: return launch_tile_flags<3>(p, groups, tiles, grid, order, log2_w, lds, s);
  }
}

hipError_t launch_rows(const StepParams& p, uint32_t groups, const Tuning& tune, hipStream_t s) {
  const bool w_pow2 = p.W <= 64 && (p.W & (p.W - 1)) == 0;
  if (tune.balanced && w_pow2 && tune.threads == 64 && tune.cols_per_lane == 1) return launch_tile(p, groups, tune, s);
  switch (tune.cols_per_lane) {
    case 1: return launch_rows_c<1>(p, groups, tune, s);
    case 4: return launch_rows_c<4>(p, groups, tune, s);
    default: return launch_rows_c<2>(p, groups, tune, s);
  }
}

}  // namespace

hipError_t launch_selector(uint64_t seed, uint32_t stream_id, uint64_t t0, uint64_t t_stride, uint32_t count, uint32_t B,
                           uint32_t k, uint8_t* mask, uint32_t* idx, hipStream_t s) {
  if (count == 0) return hipSuccess;
  const uint32_t seed_lo = static_cast<uint32_t>(seed), seed_hi = static_cast<uint32_t>(seed >> 32);
  const bool few_kept = static_cast<uint64_t>(k) * 2 < B;
  if (few_kept || idx == nullptr) {
    // fill the masks with "unchosen" (few kept) or "chosen" (most kept), then one forward evaluation per exception
    const uint8_t fill = few_kept ? 0 : 1;
    const uint32_t j_begin = few_kept ? 0u : k, j_end = few_kept ? k : B;
    const uint64_t bytes = static_cast<uint64_t>(count) * B;
    uint64_t fill_grid = (bytes / 4 + 255) / 256;
    if (fill_grid > 4096) fill_grid = 4096;
    if (fill_grid == 0) fill_grid = 1;
    hipLaunchKernelGGL(fill_bytes_kernel, dim3(static_cast<uint32_t>(fill_grid)), dim3(256), 0, s, mask, bytes, fill);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || j_end == j_begin) return err;
    const dim3 grid((j_end - j_begin + 255u) / 256u, count);
    hipLaunchKernelGGL(grbs_scatter_kernel, grid, dim3(256), 0, s, seed_lo, seed_hi, stream_id, t0, t_stride, B, j_begin,
                       j_end, static_cast<uint8_t>(1 - fill), half_bits_for(B), mask, few_kept ? idx : nullptr);
    return hipGetLastError();
  }
  const dim3 grid((B + 255u) / 256u, count);
  hipLaunchKernelGGL(grbs_select_kernel, grid, dim3(256), 0, s, seed_lo, seed_hi, stream_id, t0, t_stride, B, k,
                     half_bits_for(B), mask, idx);
  return hipGetLastError();
}

hipError_t launch_step(const StepParams& p, bool vectorised, const Tuning& tune, hipStream_t s) {
  if (!vectorised) return launch_step_range<1>(p, 0, p.d, tune, s);
  const uint64_t d4 = p.d & ~3ull;
  hipError_t err = hipSuccess;
  if (tune.variant == 0) err = launch_step_range<4>(p, 0, d4, tune, s);
  else if (d4 > 0) err = launch_rows(p, static_cast<uint32_t>(d4 / 4), tune, s);
  if (err != hipSuccess) return err;
  return launch_step_range<1>(p, d4, p.d, tune, s);   // at most 3 trailing columns
}

hipError_t launch_reset(const ResetParams& p, const uint8_t* mask, bool vectorised, hipStream_t s) {
  if (p.k == 0) return hipSuccess;
  const bool has_e = p.e != nullptr;
  uint64_t scalar_begin = 0;
  if (vectorised) {
    const uint32_t gpb = p.block / 4;
    const uint64_t total = static_cast<uint64_t>(p.k) * gpb;
    const uint32_t grid = static_cast<uint32_t>((total + 255) / 256);
    if (has_e) hipLaunchKernelGGL(cser_reset_kernel<true>, dim3(grid), dim3(256), 0, s, p, gpb, total);
    else hipLaunchKernelGGL(cser_reset_kernel<false>, dim3(grid), dim3(256), 0, s, p, gpb, total);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    scalar_begin = p.d & ~3ull;
  }
  if (scalar_begin >= p.d) return hipSuccess;
  const uint64_t n = p.d - scalar_begin;
  const uint32_t grid = static_cast<uint32_t>((n + 255) / 256);
  if (has_e) hipLaunchKernelGGL(cser_reset_scalar_kernel<true>, dim3(grid), dim3(256), 0, s, p, mask, scalar_begin, p.d);
  else hipLaunchKernelGGL(cser_reset_scalar_kernel<false>, dim3(grid), dim3(256), 0, s, p, mask, scalar_begin, p.d);
  return hipGetLastError();
}

hipError_t launch_fill_zero(float* ptr, uint64_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  uint64_t grid = (n + 255) / 256;
  if (grid > 65536) grid = 65536;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(static_cast<uint32_t>(grid)), dim3(256), 0, s, ptr, n);
  return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, uint64_t n_bytes, hipStream_t s) {
  const uint64_t n16 = n_bytes / 16;
  if (n16 == 0) return hipSuccess;
  // 256-lane workgroups, no occupancy cap: measured best for this two-stream copy (6.5 TB/s; the
  // fused-step kernel's own shape, one wavefront per workgroup with 16 per CU, copies at 5.8 TB/s)
  const uint64_t grid = (n16 + 255) / 256;
  hipLaunchKernelGGL(copy_kernel, dim3(static_cast<uint32_t>(grid)), dim3(256), 0, s, static_cast<f4*>(dst),
                     static_cast<const f4*>(src), n16);
  return hipGetLastError();
}

}  // namespace cser
