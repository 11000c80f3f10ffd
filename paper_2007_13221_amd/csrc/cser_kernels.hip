// HIP kernels of the CSER optimizer update for gfx950 (MI355X), and their launch wrappers.
//
//   grbs_select_kernel        the shared-seed block choice of the GRBS compressor (Definition 2, Section 3.3),
//   grbs_scatter_kernel       from the blocks' side (inverse permutation) or from the draws' side (forward)
//   count_chosen_kernel,      the chosen block ids of a mask in increasing order (for the reset kernel)
//   ordered_list_kernel
//   cser_step_tile_kernel     Get_p + PSync(p, C_step) + the x / e updates of Algorithm 3 in one pass, and on reset
//                             iterations the error reset as well; one-wavefront workgroups, W <= 64: the default
//   cser_step_shared_kernel   the same with W-wavefront workgroups and the worker sums staged in LDS (W <= 16);
//                             taken for the blocks that need the worker mean when they are many
//   cser_step_general_kernel  the same, one lane per column group walking all workers: any W, any block size
//   cser_reset_shared_kernel  the error-reset branch of Algorithm 3 on its own (PSync(e, C_reset), x correction)
//   cser_reset_general_kernel the same for any W and any block size
//
// The update is a pure stream over HBM (about 6 flops per 28 bytes): no matrix-core work.  States are
// worker-major rows [W][ld].  What the memory system rewards, all measured on the large workload:
//   * a wavefront should read and write ONE row, one contiguous KiB per stream, and consecutive workgroups
//     should sweep that row linearly: 6.4-6.8 TB/s for 2 to 7 streams.  Wavefronts of one workgroup (or one CU)
//     that work on W different rows at once reach 5.6-6.0, a wavefront that itself touches 2 / 4 / 8 rows per
//     access (512 / 256 / 128 contiguous bytes each) 5.6 / 5.0 / 4.4;
//   * non-temporal accesses once the state exceeds the last-level cache, and a bounded number of resident
//     wavefronts per CU (see resolve_caps).
// On a block that C_step did not choose every worker's update is independent, so the default kernel gives each
// one-wavefront workgroup one worker's row over 256 columns.  Only the chosen blocks (1 / R_step of them) need
// the worker mean, which inevitably brings W rows together: in the default kernel the W workgroups of a tile
// share that work (each takes 1/W of the tile's chosen column groups for all workers, one worker per lane group,
// the W-way sum being a fixed-order chain of wavefront shuffles).  When a large share of the blocks is chosen,
// the one-wavefront kernel takes only the blocks no compressor chose and the LDS-shared kernel, whose every access
// is still a contiguous KiB of one row, takes the others in a second launch; when nearly all are chosen the
// LDS-shared kernel runs alone (launch_step).
//
// Arithmetic, identical in every kernel: beta*m+g and beta*m_new+g are single fused multiply-adds, eta multiplies
// the rounded result, the worker sum starts from worker 0's value and adds workers 1 .. W-1 in order, the mean is
// that sum divided by W (true division).  Build with -ffp-contract=off: nothing else fuses.

#include "cser_internal.h"

#include <cmath>
#include <type_traits>

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

template <int V>
__device__ __forceinline__ Pack<V> zero_pack() {
  Pack<V> r;
#pragma unroll
  for (int c = 0; c < V; ++c) r.v[c] = 0.0f;
  return r;
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

// ==========================================================================================
// Default kernel.  One wavefront per workgroup, which owns the pair (worker i, tile of 64 column groups = 256
// columns) and plays two roles:
//   A  lane l takes column group l of the tile in worker i's row, if its block was chosen by neither
//      compressor: the purely local update  x_i -= p_i, e_i -= p_i  (28 B per element: read g, m, x, e, write
//      m, x, e), four 128-bit loads and three 128-bit stores per lane, one contiguous KiB per stream;
//   B  the tile's column groups are cut into slices of G = floor(64 / W) groups; this workgroup takes slices
//      i, i + W, ... for ALL workers: lane (j, k) = (lane / G, lane % G) holds worker j's values of group
//      slice * G + k (lanes with j >= W idle).  For groups whose block C_step chose, pbar is the in-wavefront
//      ordered sum over j divided by W:  x_j -= pbar, e_j untouched (20 B per element).  For groups C_reset
//      chose on a reset iteration the error reset follows at once, from registers:
//      ebar = ordered sum of the post-step e_j / W, x_j <- (x_j - e_j) + ebar, e_j <- +0
//      (implementation II: x_j <- ordered sum of the post-step x_j / W).
// Every workgroup of a tile thus does its share of the tile's synchronised work whatever part of the blocks is
// chosen, and each value is read and written exactly once.  Grid (tiles, W), dispatched with tiles fastest:
// the resident wavefronts sweep one worker's row through seven linear streams.
// ==========================================================================================

// Ordered worker sum inside one wavefront: every lane fetches the W values of its group k with wavefront
// shuffles and adds them in the order j = 0, 1, ..., W-1, so all W lanes of a group end up with the same bits.
// Must be called with all 64 lanes active.
__device__ __forceinline__ Pack<4> worker_sum_in_wave(const Pack<4>& v, uint32_t W, uint32_t G, uint32_t k) {
  Pack<4> sum;
#pragma unroll
  for (int c = 0; c < 4; ++c) sum.v[c] = __shfl(v.v[c], static_cast<int>(k), 64);
  for (uint32_t j = 1; j < W; ++j) {
    const int src = static_cast<int>(j * G + k);
#pragma unroll
    for (int c = 0; c < 4; ++c) sum.v[c] = sum.v[c] + __shfl(v.v[c], src, 64);
  }
  return sum;
}

template <bool NT, bool HAS_E, bool HAS_M>
__global__ __launch_bounds__(64) void cser_step_tile_kernel(StepParams a, uint32_t groups) {
  const uint32_t i = blockIdx.y, tile = blockIdx.x;   // workgroups are dispatched with x fastest: tiles of one worker's row
  const uint32_t lane = threadIdx.x;
  const uint64_t tile_first = static_cast<uint64_t>(tile) * 64u;

  // Lane l looks up the two choices for column group l of the tile; the ballots hand every lane the choices of
  // all 64 groups (bit l = group l), so role B below needs no second look-up, and a tile that neither compressor
  // touches -- the common case -- is recognised at once.
  const uint64_t qa = tile_first + lane;
  const bool live_a = qa < groups;
  const uint32_t ba = static_cast<uint32_t>(live_a ? qa : 0u) / (a.block / 4u);
  const bool step_a = live_a && a.mask[ba] != 0;
  const bool reset_a = live_a && a.reset_mask != nullptr && a.reset_mask[ba] != 0;
  const uint64_t step_bits = __ballot(step_a), reset_bits = __ballot(reset_a);

  // role A
  const bool local_a = live_a && !step_a && !reset_a;
  const uint64_t off_a = static_cast<uint64_t>(i) * a.ld + qa * 4u;
  Pack<4> ga, ma, xa, ea;
  if (local_a) {
    ga = load_pack<4, NT>(a.g + off_a);
    if constexpr (HAS_M) ma = load_pack<4, NT>(a.m + off_a);
    xa = load_pack<4, NT>(a.x + off_a);
    if constexpr (HAS_E) ea = load_pack<4, NT>(a.e + off_a);
  }
  auto finish_role_a = [&]() {
    if (local_a) {
      const Pack<4> p = local_update<4, HAS_M>(a.eta, a.beta, ga, ma);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        xa.v[c] = xa.v[c] - p.v[c];
        if constexpr (HAS_E) ea.v[c] = ea.v[c] - p.v[c];
      }
      if constexpr (HAS_M) store_pack<4, NT>(a.m + off_a, ma);
      store_pack<4, NT>(a.x + off_a, xa);
      if constexpr (HAS_E) store_pack<4, NT>(a.e + off_a, ea);
    }
  };
  if ((step_bits | reset_bits) == 0 || a.part == kPartLocal) {   // wavefront-uniform
    finish_role_a();
    return;
  }

  // role B
  const uint32_t G = 64u / a.W;                    // column groups per slice
  const uint32_t j = lane / G, k = lane - j * G;   // worker j, group k of the slice
  const uint32_t slices = (64u + G - 1u) / G;      // W when W divides 64, up to 2 W - 1 otherwise
  const float n = static_cast<float>(a.W);
  for (uint32_t slice = i; slice < slices; slice += a.W) {   // runs once when W divides 64, else once or twice
    const uint32_t within = slice * G + k;
    const bool lane_b = j < a.W && within < 64u;
    const bool step_b = lane_b && ((step_bits >> (within & 63u)) & 1u) != 0;
    const bool reset_b = lane_b && ((reset_bits >> (within & 63u)) & 1u) != 0;
    const bool sync_b = step_b || reset_b;
    const uint64_t off_b = static_cast<uint64_t>(j) * a.ld + (tile_first + within) * 4u;
    Pack<4> gb = zero_pack<4>(), mb = zero_pack<4>(), xb = zero_pack<4>(), eb = zero_pack<4>();
    if (sync_b) {
      gb = load_pack<4, NT>(a.g + off_b);
      if constexpr (HAS_M) mb = load_pack<4, NT>(a.m + off_b);
      xb = load_pack<4, NT>(a.x + off_b);
      if constexpr (HAS_E) {
        if (reset_b) eb = load_pack<4, NT>(a.e + off_b);   // e is untouched by the step on a block C_step chose
      }
    }
    if (slice == i) finish_role_a();   // role A's arithmetic, once its loads and role B's are all in flight
    if (__any(sync_b)) {   // wavefront-uniform: all 64 lanes take part in the shuffles below
      Pack<4> p = zero_pack<4>();
      if (sync_b) {
        p = local_update<4, HAS_M>(a.eta, a.beta, gb, mb);
        if constexpr (HAS_M) store_pack<4, NT>(a.m + off_b, mb);
      }
      if (__any(step_b)) {
        const Pack<4> psum = worker_sum_in_wave(p, a.W, G, k);
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
        const Pack<4> vsum = worker_sum_in_wave(v, a.W, G, k);
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
        store_pack<4, NT>(a.x + off_b, xb);
        if constexpr (HAS_E) {
          if (reset_b) store_pack<4, NT>(a.e + off_b, eb);
        }
      }
    }
  }
}

// ==========================================================================================
// LDS-shared kernels, W <= 16.  A workgroup is W wavefronts and owns a tile of 64 column groups (256 columns) of
// ALL workers: wavefront i works on worker i's row, lane l on column group l, so every global access of a
// wavefront is one contiguous KiB of one row whether the block is chosen or not.
//   block not chosen by C_step:  x_i -= p_i, e_i -= p_i, nothing is shared;
//   block chosen by C_step:      p_i goes to LDS (W KiB per workgroup), one barrier, every lane adds the W values
//                                of its column group in the order 0 .. W-1 and divides by W:  x_i -= pbar;
//   block chosen by C_reset on a reset iteration: after the step's update the post-step e_i (implementation II:
//                                x_i) is shared the same way through a second LDS area:  ebar = sum / W,
//                                x_i <- (x_i - e_i) + ebar, e_i <- +0   (II: x_i <- xbar).
// Block membership is decided per lane, so tiles cut by block boundaries (block < 256 columns) need no special
// case.  The masks are the same for every wavefront of the workgroup, hence the two `any` tests below are
// uniform over the workgroup and every wavefront reaches the same barriers.
// ==========================================================================================

// In-order sum over the workers of the values staged in LDS for this lane's column group: stage[j * 64 + lane]
// holds worker j's four values.
__device__ __forceinline__ Pack<4> worker_sum_from_lds(const f4* stage, uint32_t W, uint32_t lane) {
  f4 s = stage[lane];
  for (uint32_t j = 1; j < W; ++j) {
    const f4 v = stage[j * 64u + lane];
    s.x = s.x + v.x; s.y = s.y + v.y; s.z = s.z + v.z; s.w = s.w + v.w;
  }
  Pack<4> r;
  r.v[0] = s.x; r.v[1] = s.y; r.v[2] = s.z; r.v[3] = s.w;
  return r;
}

__device__ __forceinline__ f4 as_f4(const Pack<4>& p) {
  f4 t;
  t.x = p.v[0]; t.y = p.v[1]; t.z = p.v[2]; t.w = p.v[3];
  return t;
}

template <bool NT, bool HAS_E, bool HAS_M>
__global__ __launch_bounds__(1024) void cser_step_shared_kernel(StepParams a, uint32_t groups) {
  extern __shared__ f4 stage[];
  const uint32_t lane = threadIdx.x & 63u, i = threadIdx.x >> 6;
  const uint64_t q = static_cast<uint64_t>(blockIdx.x) * 64u + lane;
  bool live = q < groups;
  const uint32_t b = static_cast<uint32_t>(live ? q : 0u) / (a.block / 4u);
  const bool step_c = live && a.mask[b] != 0;
  const bool reset_c = live && a.reset_mask != nullptr && a.reset_mask[b] != 0;
  if (a.part == kPartSynchronised) {
    // the blocks neither compressor chose have been updated by the one-wavefront kernel.  The masks are the same
    // for every wavefront of the workgroup, so either all of them leave here or none does.
    live = live && (step_c || reset_c);
    if (!__any(live)) return;
  }
  const bool touches_e = HAS_E && live && (!step_c || reset_c);   // e is untouched by the step on a block C_step chose
  const uint64_t off = static_cast<uint64_t>(i) * a.ld + q * 4u;
  Pack<4> g = zero_pack<4>(), m = zero_pack<4>(), x = zero_pack<4>(), e = zero_pack<4>();
  if (live) {
    g = load_pack<4, NT>(a.g + off);
    if constexpr (HAS_M) m = load_pack<4, NT>(a.m + off);
    x = load_pack<4, NT>(a.x + off);
  }
  if (touches_e) e = load_pack<4, NT>(a.e + off);
  Pack<4> p = local_update<4, HAS_M>(a.eta, a.beta, g, m);
  if constexpr (HAS_M) {
    if (live) store_pack<4, NT>(a.m + off, m);
  }
  const float n = static_cast<float>(a.W);
  if (__any(step_c)) {
    if (step_c) stage[i * 64u + lane] = as_f4(p);
    __syncthreads();
    if (step_c) {
      const Pack<4> psum = worker_sum_from_lds(stage, a.W, lane);
#pragma unroll
      for (int c = 0; c < 4; ++c) p.v[c] = psum.v[c] / n;      // p' = pbar, r = 0
    }
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    x.v[c] = x.v[c] - p.v[c];
    if constexpr (HAS_E) {
      if (!step_c) e.v[c] = e.v[c] - p.v[c];                    // r = p off the blocks C_step chose
    }
  }
  if (a.reset_mask != nullptr && __any(reset_c)) {
    f4* stage2 = stage + a.W * 64u;
    if (reset_c) stage2[i * 64u + lane] = as_f4(HAS_E ? e : x);
    __syncthreads();
    if (reset_c) {
      const Pack<4> vsum = worker_sum_from_lds(stage2, a.W, lane);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float mean = vsum.v[c] / n;
        if constexpr (HAS_E) {
          x.v[c] = (x.v[c] - e.v[c]) + mean;
          e.v[c] = 0.0f;
        } else {
          x.v[c] = mean;
        }
      }
    }
  }
  if (live) store_pack<4, NT>(a.x + off, x);
  if (touches_e) store_pack<4, NT>(a.e + off, e);
}

// Error reset on its own (cser_error_reset), same shape: a workgroup of W wavefronts owns 64 column groups of
// the blocks listed in idx, wavefront i reads worker i's e and x once (one contiguous KiB each when the block has
// at least 256 columns), the worker sum goes through LDS, and x and e are written once:
//   ebar = (e_0 + e_1 + ... + e_{W-1}) / W ;  x_i <- (x_i - e_i) + ebar ;  e_i <- +0
// (implementation II, no e:  x_i <- (x_0 + ... + x_{W-1}) / W).  idx is in increasing order, so consecutive
// workgroups sweep the rows forwards (a list in draw order costs 20 % of the bandwidth).
template <bool NT, bool HAS_E>
__global__ __launch_bounds__(1024) void cser_reset_shared_kernel(ResetParams a, uint32_t groups_per_block,
                                                                  uint64_t total_groups) {
  extern __shared__ f4 stage[];
  const uint32_t lane = threadIdx.x & 63u, i = threadIdx.x >> 6;
  const uint64_t q = static_cast<uint64_t>(blockIdx.x) * 64u + lane;
  bool live = q < total_groups;
  const uint32_t j = static_cast<uint32_t>((live ? q : 0u) / groups_per_block);
  const uint32_t within = static_cast<uint32_t>((live ? q : 0u) - static_cast<uint64_t>(j) * groups_per_block);
  const uint64_t col = static_cast<uint64_t>(a.idx[j]) * a.block + static_cast<uint64_t>(within) * 4u;
  live = live && col + 4u <= a.d;   // ragged last block; a trailing partial group goes to the element-wise kernel
  const uint64_t off = static_cast<uint64_t>(i) * a.ld + col;
  Pack<4> x = zero_pack<4>(), e = zero_pack<4>();
  if (live) {
    if constexpr (HAS_E) e = load_pack<4, NT>(a.e + off);
    x = load_pack<4, NT>(a.x + off);
  }
  stage[i * 64u + lane] = as_f4(HAS_E ? e : x);
  __syncthreads();
  if (live) {
    const Pack<4> vsum = worker_sum_from_lds(stage, a.W, lane);
    const float n = static_cast<float>(a.W);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float mean = vsum.v[c] / n;
      if constexpr (HAS_E) {
        x.v[c] = (x.v[c] - e.v[c]) + mean;
        e.v[c] = 0.0f;
      } else {
        x.v[c] = mean;
      }
    }
    store_pack<4, NT>(a.x + off, x);
    if constexpr (HAS_E) store_pack<4, NT>(a.e + off, e);
  }
}

// ==========================================================================================
// General kernels: one lane per group of V columns walks the worker axis itself (a private chain of adds in
// registers).  Any W, any block size (V = 1 when block is not a multiple of 4 columns, and for the up to 3
// trailing columns of a d that is not).  U workers are processed per batch: all their loads are issued before
// any arithmetic.
//   block not chosen by C_step:  C(p_i) = 0 on every worker, so the mean is 0, p'_i = r_i = p_i:
//                                x_i -= p_i, e_i -= p_i
//   block chosen:                r_i = 0, p'_i = mean_j p_j:  x_i -= pbar, e_i untouched
// ==========================================================================================
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
    for (int c = 0; c < V; ++c) sum.v[c] = (i0 + u == 0u) ? p.v[c] : sum.v[c] + p.v[c];   // workers in order 0, 1, ...
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
    Pack<V> sum = zero_pack<V>();
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

// Reset iterations (t mod H = 0) with the reset fused into the step: the V columns at `col` belong
// to a block C_reset chose, so after the step's own update the error reset follows at once,
//   ebar = (e'_0 + ... + e'_{W-1}) / W ;  x_i <- (x'_i - e'_i) + ebar ;  e_i <- +0
// (implementation II: x_i <- (x'_0 + ... + x'_{W-1}) / W), where x', e' are the values after the
// step.  Every operation and its order are those of running the step and then the reset; x and e just travel
// through registers instead of memory.  A worker's update p_i is recomputed from g_i and the old m_i in each
// pass (m is stored only in the last), so no pass reads what an earlier pass wrote.  Plain (temporal) accesses:
// the re-reads are meant to hit in L2.
template <int V, bool HAS_E, bool HAS_M>
__device__ __forceinline__ void step_and_reset_columns(const StepParams& a, uint64_t col, bool step_chosen) {
  const float n = static_cast<float>(a.W);
  const Pack<V> zero = zero_pack<V>();
  Pack<V> pbar = zero, sum = zero, mean;
  if (step_chosen) {   // pbar = mean_i p_i
    Pack<V> psum = zero;
    for (uint32_t i = 0; i < a.W; ++i) {
      const uint64_t off = static_cast<uint64_t>(i) * a.ld + col;
      const Pack<V> g = load_pack<V, false>(a.g + off);
      Pack<V> m = zero;
      if constexpr (HAS_M) m = load_pack<V, false>(a.m + off);
      const Pack<V> p = local_update<V, HAS_M>(a.eta, a.beta, g, m);
#pragma unroll
      for (int c = 0; c < V; ++c) psum.v[c] = i == 0u ? p.v[c] : psum.v[c] + p.v[c];
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
    for (int c = 0; c < V; ++c) sum.v[c] = i == 0u ? v.v[c] : sum.v[c] + v.v[c];
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

// Columns [col_begin, col_begin + groups * V) in groups of V.  With V = 4, col_begin is 0 and block is a
// multiple of 4, so a group never straddles two blocks.
template <int V, bool NT, bool HAS_E, bool HAS_M>
__global__ __launch_bounds__(256) void cser_step_general_kernel(StepParams a, uint64_t col_begin, uint32_t groups) {
  const uint64_t q = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (q >= groups) return;
  const uint64_t col = col_begin + q * V;
  uint32_t b;
  if constexpr (V == 4) b = static_cast<uint32_t>(q) / (a.block / 4u);
  else b = static_cast<uint32_t>(col / a.block);
  const bool step_chosen = a.mask[b] != 0;
  const bool reset_chosen = a.reset_mask != nullptr && a.reset_mask[b] != 0;
  if (a.part == kPartSynchronised && !step_chosen && !reset_chosen) return;   // updated by the one-wavefront kernel
  if (reset_chosen) step_and_reset_columns<V, HAS_E, HAS_M>(a, col, step_chosen);
  else step_columns<V, 4, NT, HAS_E, HAS_M>(a, col, step_chosen);
}

// Error reset on the V columns at `col` of a chosen block; the second pass re-reads e_i (the lines were just
// fetched by this lane, so they come from L2).
template <int V, bool HAS_E>
__device__ __forceinline__ void reset_columns(const ResetParams& a, uint64_t col) {
  float* src = HAS_E ? a.e : a.x;
  Pack<V> sum = zero_pack<V>();
  for (uint32_t i = 0; i < a.W; ++i) {
    const Pack<V> v = load_pack<V, false>(src + static_cast<uint64_t>(i) * a.ld + col);
#pragma unroll
    for (int c = 0; c < V; ++c) sum.v[c] = i == 0u ? v.v[c] : sum.v[c] + v.v[c];
  }
  const float n = static_cast<float>(a.W);
  const Pack<V> zero = zero_pack<V>();
  Pack<V> mean;
#pragma unroll
  for (int c = 0; c < V; ++c) mean.v[c] = sum.v[c] / n;
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

// V = 4: one lane per 4-column group of a listed block.  V = 1: one lane per column of [col_begin, col_begin +
// total), chosen or not by the mask (any alignment, any block size).
template <int V, bool HAS_E>
__global__ __launch_bounds__(256) void cser_reset_general_kernel(ResetParams a, const uint8_t* mask, uint32_t groups_per_block,
                                                                  uint64_t total, uint64_t col_begin) {
  const uint64_t q = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (q >= total) return;
  if constexpr (V == 4) {
    const uint32_t j = static_cast<uint32_t>(q / groups_per_block);
    const uint32_t within = static_cast<uint32_t>(q - static_cast<uint64_t>(j) * groups_per_block);
    const uint64_t col = static_cast<uint64_t>(a.idx[j]) * a.block + static_cast<uint64_t>(within) * 4u;
    if (col + 4u > a.d) return;   // ragged last block; a trailing partial group goes to the V = 1 launch
    reset_columns<4, HAS_E>(a, col);
  } else {
    const uint64_t col = col_begin + q;
    if (mask[col / a.block] == 0) return;
    reset_columns<1, HAS_E>(a, col);
  }
}

// ==========================================================================================
// Block selector.  All workers must pick the same k of the B blocks from a shared seed
// (Definition 2).  The choice is {pi(0), ..., pi(k-1)} for a keyed permutation pi of [0, B):
// block b is chosen iff pi^-1(b) < k, which every block can decide for itself -- no sort, no
// atomics, one thread per block.
//
// pi: 8-round balanced Feistel network on 2h bits (2^(2h) >= B), round function = low h bits of
// word 0 of Philox-4x32-10 (Salmon et al., SC'11) keyed by the seed with counter
// (half, stream*65536 + round, t_lo, t_hi); values >= B are walked through the network again
// (cycle walking).
// ==========================================================================================
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

// Inverse form.  blockIdx.y selects the iteration t0 + blockIdx.y * t_stride (the choice is a pure function of
// t, so several iterations can be drawn ahead in one launch); its mask goes to mask + blockIdx.y * B.  idx may
// be null; when given it is only meaningful for a launch with gridDim.y == 1.
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

// The block ids b with mask[b] != 0 in increasing order, out[0 .. k): two launches over the same decomposition.
// The mask is cut into chunks of `chunk` bytes (a multiple of 4096, at most 1024 chunks), one workgroup of 256
// lanes per chunk, each lane owning chunk / 256 consecutive bytes.  count_chosen_kernel writes the number of
// chosen blocks of every chunk; ordered_list_kernel adds up the counts of the chunks before its own, scans its
// lanes' counts and writes the ids.  `k` bounds the writes (the mask holds exactly k chosen blocks by construction).
__device__ __forceinline__ uint32_t count_nonzero_bytes(const uint8_t* mask, uint64_t begin, uint64_t end) {
  uint32_t c = 0;
  uint64_t b = begin;
  for (; b + 16 <= end; b += 16) {   // begin is a multiple of 16 and the mask is 16-byte aligned
    const uint4 w = *reinterpret_cast<const uint4*>(mask + b);
    const uint32_t words[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int s = 0; s < 32; s += 8) c += ((words[i] >> s) & 0xFFu) != 0 ? 1u : 0u;
    }
  }
  for (; b < end; ++b) c += mask[b] != 0 ? 1u : 0u;
  return c;
}

__device__ __forceinline__ uint32_t workgroup_inclusive_scan_256(uint32_t value, uint32_t* shared) {
  const uint32_t tid = threadIdx.x;
  shared[tid] = value;
  __syncthreads();
  for (uint32_t step = 1; step < 256u; step <<= 1) {
    const uint32_t add = tid >= step ? shared[tid - step] : 0u;
    __syncthreads();
    shared[tid] += add;
    __syncthreads();
  }
  return shared[tid];
}

__global__ __launch_bounds__(256) void count_chosen_kernel(const uint8_t* mask, uint32_t B, uint32_t chunk, uint32_t* counts) {
  __shared__ uint32_t shared[256];
  const uint64_t per = chunk / 256u;
  const uint64_t begin = static_cast<uint64_t>(blockIdx.x) * chunk + threadIdx.x * per;
  const uint64_t b0 = begin < B ? begin : B, b1 = begin + per < B ? begin + per : B;
  const uint32_t total = workgroup_inclusive_scan_256(count_nonzero_bytes(mask, b0, b1), shared);
  if (threadIdx.x == 255u) counts[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void ordered_list_kernel(const uint8_t* mask, uint32_t B, uint32_t chunk, const uint32_t* counts,
                                                            uint32_t k, uint32_t* out) {
  __shared__ uint32_t shared[256];
  const uint32_t tid = threadIdx.x;
  uint32_t before = 0;   // chosen blocks in the chunks before this one: every lane adds up a stride of the counts
  for (uint32_t c = tid; c < blockIdx.x; c += 256u) before += counts[c];
  (void)workgroup_inclusive_scan_256(before, shared);   // leaves the total in shared[255]
  const uint32_t chunk_base = shared[255];
  __syncthreads();                                       // everyone has read it before `shared` is used again
  const uint64_t per = chunk / 256u;
  const uint64_t begin = static_cast<uint64_t>(blockIdx.x) * chunk + tid * per;
  const uint64_t b0 = begin < B ? begin : B, b1 = begin + per < B ? begin + per : B;
  const uint32_t mine = count_nonzero_bytes(mask, b0, b1);
  uint32_t pos = chunk_base + workgroup_inclusive_scan_256(mine, shared) - mine;
  for (uint64_t b = b0; b < b1; ++b) {
    if (mask[b] != 0 && pos < k) out[pos++] = static_cast<uint32_t>(b);
  }
}

__global__ __launch_bounds__(256) void fill_bytes_kernel(uint8_t* p, uint64_t n, uint8_t value) {
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  const uint64_t n4 = n / 4;   // p is at least 4-byte aligned
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

// Calls f(NT, HAS_E, HAS_M) with the three flags as compile-time constants.
template <class F>
auto with_flags(bool nt, bool has_e, bool has_m, F&& f) {
  auto pick_m = [&](auto NT, auto E) { return has_m ? f(NT, E, std::true_type{}) : f(NT, E, std::false_type{}); };
  auto pick_e = [&](auto NT) { return has_e ? pick_m(NT, std::true_type{}) : pick_m(NT, std::false_type{}); };
  return nt ? pick_e(std::true_type{}) : pick_e(std::false_type{});
}

template <int V>
hipError_t launch_general(const StepParams& p, uint64_t col_begin, uint64_t col_end, bool nt, hipStream_t s) {
  if (col_end <= col_begin) return hipSuccess;
  const uint64_t groups64 = (col_end - col_begin) / V;
  if (groups64 == 0) return hipSuccess;
  const uint32_t groups = static_cast<uint32_t>(groups64);
  const dim3 grid(static_cast<uint32_t>((groups64 + 255) / 256)), block(256);
  return with_flags(nt, p.e != nullptr, p.m != nullptr, [&](auto NT, auto E, auto M) {
    hipLaunchKernelGGL((cser_step_general_kernel<V, decltype(NT)::value, decltype(E)::value, decltype(M)::value>), grid, block,
                       0, s, p, col_begin, groups);
    return hipGetLastError();
  });
}

hipError_t launch_tile(const StepParams& p, uint32_t groups, bool nt, uint32_t lds, hipStream_t s) {
  const uint64_t tiles64 = (static_cast<uint64_t>(groups) + 63) / 64;
  if (tiles64 * p.W > 0x7FFFFFFFull || p.W > 65535u) return hipErrorInvalidConfiguration;   // launch_step never asks for such a grid
  const dim3 grid(static_cast<uint32_t>(tiles64), p.W), block(64);
  return with_flags(nt, p.e != nullptr, p.m != nullptr, [&](auto NT, auto E, auto M) {
    hipLaunchKernelGGL((cser_step_tile_kernel<decltype(NT)::value, decltype(E)::value, decltype(M)::value>), grid, block, lds, s,
                       p, groups);
    return hipGetLastError();
  });
}

hipError_t launch_shared(const StepParams& p, uint32_t groups, bool nt, uint32_t lds, hipStream_t s) {
  const dim3 grid((groups + 63u) / 64u), block(64u * p.W);
  return with_flags(nt, p.e != nullptr, p.m != nullptr, [&](auto NT, auto E, auto M) {
    hipLaunchKernelGGL((cser_step_shared_kernel<decltype(NT)::value, decltype(E)::value, decltype(M)::value>), grid, block, lds,
                       s, p, groups);
    return hipGetLastError();
  });
}

// Smallest dynamic-LDS request (a multiple of 256 bytes, at least `needed`, at most 64 KiB) under which the
// runtime's occupancy calculator fits no more than `want` workgroups of `threads` lanes of kernel `fn` on a CU;
// want = 0 asks for no cap.  *resident receives what the calculator reports for the request returned.
hipError_t cap_by_lds(const void* fn, uint32_t threads, uint32_t needed, uint32_t want, uint32_t* lds, uint32_t* resident) {
  auto fits = [&](uint32_t bytes, int* n) {
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(n, fn, static_cast<int>(threads), bytes);
  };
  int n = 0;
  uint32_t lo = (needed + 255u) / 256u, hi = 65536u / 256u;   // in units of 256 bytes
  hipError_t err = fits(needed, &n);
  if (err != hipSuccess) return err;
  if (want == 0 || static_cast<uint32_t>(n) <= want) {
    *lds = needed;
    *resident = static_cast<uint32_t>(n);
    return hipSuccess;
  }
  err = fits(hi * 256u, &n);
  if (err != hipSuccess) return err;
  if (static_cast<uint32_t>(n) > want) {   // even the largest request leaves more than wanted: take it
    *lds = hi * 256u;
    *resident = static_cast<uint32_t>(n);
    return hipSuccess;
  }
  if (lo > 0) lo -= 1;   // fits(lo) > want holds for the request `needed`, hence for anything below it
  while (hi - lo > 1) {   // invariant: fits(lo) > want >= fits(hi)
    const uint32_t mid = (lo + hi) / 2;
    err = fits(mid * 256u, &n);
    if (err != hipSuccess) return err;
    if (static_cast<uint32_t>(n) > want) lo = mid;
    else hi = mid;
  }
  err = fits(hi * 256u, &n);
  if (err != hipSuccess) return err;
  *lds = hi * 256u;
  *resident = static_cast<uint32_t>(n);
  return hipSuccess;
}

}  // namespace

// Residency: what the memory system rewards is about 48 KiB of loads in flight per CU.  Measured on the large workload
// (R_step 256, 8, 4, 2), the one-wavefront kernel is fastest with 10-13 resident wavefronts per CU when a wavefront
// has 4 load streams (g, m, x, e; 16: 0.5-2 % slower, 8: 3-5 % slower, uncapped, where 28 fit: 5 % slower), 14-20 with
// 3, uncapped with 2 (there a cap of 20 costs 4-14 %); the LDS-shared kernels with about 24 wavefronts per CU.
hipError_t resolve_caps(uint32_t W, bool has_e, bool has_m, bool nontemporal, const Tuning& tune, Caps* out) {
  *out = Caps();
  hipError_t err = hipSuccess;
  {   // the one-wavefront kernel: any W (beyond 64 workers it only ever takes the blocks no compressor chose)
    const int streams = 2 + (has_e ? 1 : 0) + (has_m ? 1 : 0);
    const uint32_t want = tune.tile_waves_per_cu >= 0 ? static_cast<uint32_t>(tune.tile_waves_per_cu)
                                                      : (streams >= 4 ? 12u : (streams == 3 ? 18u : 0u));
    const void* fn = with_flags(nontemporal, has_e, has_m, [](auto NT, auto E, auto M) {
      return reinterpret_cast<const void*>(&cser_step_tile_kernel<decltype(NT)::value, decltype(E)::value, decltype(M)::value>);
    });
    err = cap_by_lds(fn, 64, 0, want, &out->tile_lds, &out->tile_resident);
    if (err != hipSuccess) return err;
  }
  if (W <= 16) {
    uint32_t want = tune.shared_groups_per_cu >= 0 ? static_cast<uint32_t>(tune.shared_groups_per_cu) : 24u / W;
    if (tune.shared_groups_per_cu < 0 && want < 2) want = 2;
    const void* fn = with_flags(nontemporal, has_e, has_m, [](auto NT, auto E, auto M) {
      return reinterpret_cast<const void*>(&cser_step_shared_kernel<decltype(NT)::value, decltype(E)::value, decltype(M)::value>);
    });
    err = cap_by_lds(fn, 64 * W, W * 1024u, want, &out->shared_lds, &out->shared_resident);
    if (err != hipSuccess) return err;
    err = cap_by_lds(fn, 64 * W, 2u * W * 1024u, want, &out->shared_reset_lds, &out->shared_reset_resident);
    if (err != hipSuccess) return err;
    const void* rfn = nontemporal ? (has_e ? reinterpret_cast<const void*>(&cser_reset_shared_kernel<true, true>)
                                          : reinterpret_cast<const void*>(&cser_reset_shared_kernel<true, false>))
                                  : (has_e ? reinterpret_cast<const void*>(&cser_reset_shared_kernel<false, true>)
                                          : reinterpret_cast<const void*>(&cser_reset_shared_kernel<false, false>));
    err = cap_by_lds(rfn, 64 * W, W * 1024u, want, &out->reset_lds, &out->reset_resident);
  }
  return err;
}

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

uint32_t ordered_list_chunk(uint32_t B) {
  uint64_t chunk = 4096;   // bytes of the mask per workgroup: at most 1024 workgroups
  while ((static_cast<uint64_t>(B) + chunk - 1) / chunk > 1024) chunk *= 2;
  return static_cast<uint32_t>(chunk);
}

hipError_t launch_ordered_list(const uint8_t* mask, uint32_t B, uint32_t k, uint32_t* counts, uint32_t* idx_sorted,
                               hipStream_t s) {
  if (k == 0) return hipSuccess;
  const uint32_t chunk = ordered_list_chunk(B);
  const dim3 grid(static_cast<uint32_t>((static_cast<uint64_t>(B) + chunk - 1) / chunk)), block(256);
  hipLaunchKernelGGL(count_chosen_kernel, grid, block, 0, s, mask, B, chunk, counts);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(ordered_list_kernel, grid, block, 0, s, mask, B, chunk, counts, k, idx_sorted);
  return hipGetLastError();
}

// The one-wavefront kernel's grid is (tiles, W): at most 65,535 workers and 2^31 - 1 workgroups.
bool tile_grid_fits(uint64_t d, uint32_t W) {
  const uint64_t tiles = (d / 4 + 63) / 64;
  return W <= 65535u && tiles * W <= 0x7FFFFFFFull;
}

int choose_step_kernel(uint64_t d, uint32_t W, uint32_t block, bool vectorised, double sync_share, const Tuning& tune) {
  if (!vectorised) return kKernelGeneral;
  int kernel = tune.kernel;
  if (kernel == kKernelTile && W > 64) kernel = kKernelAuto;       // its synchronised path gives each of W lane groups a run of 64 / W column groups
  if (kernel == kKernelShared && W > 16) kernel = kKernelAuto;     // W wavefronts per workgroup
  if (kernel == kKernelSplit && !tile_grid_fits(d, W)) kernel = kKernelAuto;
  if (kernel != kKernelAuto) return kernel;
  // By the share of the blocks that need the worker mean in this launch (measured on the large workload;
  // algorithmic TB/s of the blocks concerned, W = 8):
  //   * the one-wavefront kernel sweeps the other blocks at 6.5-6.7 but handles the synchronised ones at 5
  //     (1-3 when 64 / W column groups are not a run of 64 bytes or more: W = 3, 6, 12 and everything from 16 on):
  //     best while they are few;
  //   * the LDS-shared kernel moves the synchronised blocks at 6.0-6.3 and the others, W rows at a time from
  //     one CU, at 5.5-6.0: best when nearly every block is synchronised;
  //   * in between, each kernel does what it is good at: the one-wavefront kernel takes the blocks neither
  //     compressor chose, then the LDS-shared kernel the others.  Its workgroups that find nothing to do cost
  //     about 50 us per 100,000 tiles, which sets the lower end of the range;
  //   * beyond 16 workers the general kernel (5 TB/s on anything) stands in for the LDS-shared one.
  // Break-even points measured for W = 3, 6, 8, 12, 16, 24, 32, 64, 96 at R_step = 2 .. 256.
  // The pair needs tiles that are synchronised as a whole or not at all: with blocks shorter than a tile (256
  // columns) most tiles hold both kinds, both launches would visit them, and one kernel on its own is faster
  // (block 64, R_step 2: pair 0.97 ms, LDS-shared kernel 0.83, one-wavefront kernel 0.86).
  const bool wide_runs = W == 1 || W == 2 || W == 4 || W == 8;
  const double blocks_per_tile = block >= 256u ? 1.0 : 256.0 / static_cast<double>(block);
  const double mixed_tiles = 1.0 - std::pow(sync_share, blocks_per_tile) - std::pow(1.0 - sync_share, blocks_per_tile);
  if (W <= 16) {
    if (sync_share >= 0.9) return kKernelShared;
    if (mixed_tiles > 0.25 && sync_share >= (wide_runs ? 0.5 : 0.1)) return kKernelShared;
    if (mixed_tiles <= 0.25 && sync_share >= (wide_runs ? 0.4 : 0.1)) return kKernelSplit;
    return kKernelTile;
  }
  if (!tile_grid_fits(d, W) || sync_share >= 0.9) return kKernelGeneral;
  if (W > 64 || sync_share > 0.0) {   // beyond 16 workers the pair is never slower (W = 24, 32, 64 at R_step 256: +0.3 .. +3 %)
    return mixed_tiles <= 0.25 ? kKernelSplit : kKernelGeneral;
  }
  return kKernelTile;
}

hipError_t launch_step(const StepParams& p_in, bool vectorised, bool nontemporal, const Tuning& tune, const Caps& caps,
                       double sync_share, int* used, hipStream_t s) {
  StepParams p = p_in;
  p.part = kPartAll;
  const int kernel = choose_step_kernel(p.d, p.W, p.block, vectorised, sync_share, tune);
  if (used) *used = kernel;
  if (!vectorised) return launch_general<1>(p, 0, p.d, nontemporal, s);
  const uint64_t d4 = p.d & ~3ull;
  hipError_t err = hipSuccess;
  if (d4 > 0) {
    const uint32_t groups = static_cast<uint32_t>(d4 / 4);
    const uint32_t shared_lds = p.reset_mask != nullptr ? caps.shared_reset_lds : caps.shared_lds;
    if (kernel == kKernelTile) {
      err = launch_tile(p, groups, nontemporal, caps.tile_lds, s);
    } else if (kernel == kKernelShared) {
      err = launch_shared(p, groups, nontemporal, shared_lds, s);
    } else if (kernel == kKernelSplit) {
      p.part = kPartLocal;
      err = launch_tile(p, groups, nontemporal, caps.tile_lds, s);
      p.part = kPartSynchronised;
      if (err == hipSuccess) {
        if (p.W <= 16) err = launch_shared(p, groups, nontemporal, shared_lds, s);
        else err = launch_general<4>(p, 0, d4, nontemporal, s);
      }
      p.part = kPartAll;
    } else {
      err = launch_general<4>(p, 0, d4, nontemporal, s);
    }
  }
  if (err != hipSuccess) return err;
  return launch_general<1>(p, d4, p.d, nontemporal, s);   // at most 3 trailing columns
}

hipError_t launch_reset(const ResetParams& p, const uint8_t* mask, bool vectorised, bool nontemporal, const Tuning& tune,
                        const Caps& caps, hipStream_t s) {
  if (p.k == 0) return hipSuccess;
  const bool has_e = p.e != nullptr;
  uint64_t scalar_begin = 0;
  if (vectorised) {
    const uint32_t gpb = p.block / 4;
    const uint64_t total = static_cast<uint64_t>(p.k) * gpb;
    if (p.W <= 16 && tune.kernel != kKernelGeneral) {
      const dim3 grid(static_cast<uint32_t>((total + 63) / 64)), block(64u * p.W);
      const uint32_t lds = caps.reset_lds > p.W * 1024u ? caps.reset_lds : p.W * 1024u;
      if (nontemporal) {
        if (has_e) hipLaunchKernelGGL((cser_reset_shared_kernel<true, true>), grid, block, lds, s, p, gpb, total);
        else hipLaunchKernelGGL((cser_reset_shared_kernel<true, false>), grid, block, lds, s, p, gpb, total);
      } else {
        if (has_e) hipLaunchKernelGGL((cser_reset_shared_kernel<false, true>), grid, block, lds, s, p, gpb, total);
        else hipLaunchKernelGGL((cser_reset_shared_kernel<false, false>), grid, block, lds, s, p, gpb, total);
      }
    } else {
      const dim3 grid(static_cast<uint32_t>((total + 255) / 256)), block(256);
      if (has_e) hipLaunchKernelGGL((cser_reset_general_kernel<4, true>), grid, block, 0, s, p, mask, gpb, total, 0);
      else hipLaunchKernelGGL((cser_reset_general_kernel<4, false>), grid, block, 0, s, p, mask, gpb, total, 0);
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    scalar_begin = p.d & ~3ull;
  }
  if (scalar_begin >= p.d) return hipSuccess;
  const uint64_t n = p.d - scalar_begin;
  const dim3 grid(static_cast<uint32_t>((n + 255) / 256)), block(256);
  if (has_e) hipLaunchKernelGGL((cser_reset_general_kernel<1, true>), grid, block, 0, s, p, mask, 0, n, scalar_begin);
  else hipLaunchKernelGGL((cser_reset_general_kernel<1, false>), grid, block, 0, s, p, mask, 0, n, scalar_begin);
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
  // 256-lane workgroups, no occupancy cap: measured best for this two-stream copy
  const uint64_t grid = (n16 + 255) / 256;
  hipLaunchKernelGGL(copy_kernel, dim3(static_cast<uint32_t>(grid)), dim3(256), 0, s, static_cast<f4*>(dst),
                     static_cast<const f4*>(src), n16);
  return hipGetLastError();
}

}  // namespace cser
