// CSER reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
//
// A plain, slow, single-threaded CPU statement of what the CSER optimizer update
// computes, written from the paper (arxiv 2007.13221).  Only the test-suite, the
// smoke check and the benchmark's cpu-baseline leg may load it; the GPU library
// shares no code, header, table or helper with this file.
//
// What is implemented, and from where:
//   * PSync                         -- Algorithm "Partial Synchronization (PSync)" (Section 3.1)
//   * GRBS compressor               -- Definition 2 (Section 3.3): partition into blocks, the same
//                                      randomly picked blocks on every worker, zero elsewhere
//   * M-CSER, implementation I      -- Algorithm 3 (Section 3.2); with beta = 0 it is Algorithm 2
//   * CSER, implementation II       -- Appendix A.4 (no residual buffer; PSync acts on x)
//   * Get_p                         -- Appendix A.4, "Calculate update on worker i"
//
// The routines follow the algorithm boxes statement by statement on whole vectors
// (restricted to a column range when the caller simulates a slice of the blocks);
// there is no fusion of statements, and PSync really forms C(v), r = v - C(v), the worker
// mean of C(v), and mean + r for every column.  The one place where chosen and unchosen
// blocks are told apart is the model correction of the error reset, x <- x - e + e': where
// the block is not chosen e' is identically e, and x is left untouched instead of being
// sent through (x - e) + e, which is the identity only in exact arithmetic.
//
// Arithmetic contract (the paper fixes no precision; these are this build's readings):
//   * `real` is float (the resident-state precision) or double (a truth run used to
//     bound the float run's rounding error).
//   * beta*m + g and beta*m_new + g are each one fused multiply-add; eta multiplies
//     the rounded result.
//   * the worker mean is the left-to-right sum over i = 0..n-1 divided by n.
//   * the shared-seed block choice is a keyed permutation of the block ids (below);
//     the paper only asks that all workers draw the same random blocks.
//
// Parity status: the selector's concrete index lists and the bit values of the states are
// fixed by no printed number in the paper ("parity unpinned" at the level of literal
// values); every routine is pinned instead by invariants, closed forms, special cases and
// exact brute force in tests/test_oracle_*.py.

#include <cmath>
#include <cstddef>
#include <cstdint>
#include <vector>

namespace {

// ---------------------------------------------------------------------------------
// Philox-4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
// 1, 2, 3", SC'11): counter-based generator, 4 x 32-bit counter, 2 x 32-bit key.
// ---------------------------------------------------------------------------------
void philox4x32_10(const uint32_t counter[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t mult_a = 0xD2511F53u;
  const uint64_t mult_b = 0xCD9E8D57u;
  const uint32_t weyl_a = 0x9E3779B9u;
  const uint32_t weyl_b = 0xBB67AE85u;
  uint32_t c0 = counter[0], c1 = counter[1], c2 = counter[2], c3 = counter[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += weyl_a;
      k1 += weyl_b;
    }
    const uint64_t prod_a = mult_a * c0;
    const uint64_t prod_b = mult_b * c2;
    const uint32_t n0 = static_cast<uint32_t>(prod_b >> 32) ^ c1 ^ k0;
    const uint32_t n1 = static_cast<uint32_t>(prod_b);
    const uint32_t n2 = static_cast<uint32_t>(prod_a >> 32) ^ c3 ^ k1;
    const uint32_t n3 = static_cast<uint32_t>(prod_a);
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// ---------------------------------------------------------------------------------
// Shared-seed block choice (Definition 2: every worker picks the same B/R random blocks).
//
// A keyed permutation pi of [0, B), a pure function of (seed, stream, t):
//   * width: n = the smallest integer with 2^n >= B, raised to at least 2; h = ceil(n / 2);
//     the network permutes the 2h-bit integers (fewer than 4B of them once B >= 2);
//   * 8 balanced Feistel rounds (L, R) -> (R, L xor F(round, R)),
//     F = low h bits of word 0 of Philox-4x32-10 with
//     counter (R, stream * 65536 + round, low32(t), high32(t)) and key (low32(seed), high32(seed));
//   * cycle-walking: pi(v) is the first iterate of the network, applied to v at least once,
//     that is < B.
// The selection for (seed, stream, t) is { pi(0), ..., pi(k-1) }: exactly k distinct blocks.
// ---------------------------------------------------------------------------------
const int kFeistelRounds = 8;

struct BlockPermutation {
  uint64_t seed;
  uint32_t stream;
  uint64_t t;
  uint64_t B;
  uint32_t half_bits;

  BlockPermutation(uint64_t seed_, uint32_t stream_, uint64_t t_, uint64_t B_)
      : seed(seed_), stream(stream_), t(t_), B(B_) {
    uint32_t bits = 0;
    while ((uint64_t{1} << bits) < B) ++bits;
    if (bits < 2) bits = 2;
    half_bits = (bits + 1) / 2;
  }

  uint32_t round_function(uint32_t round, uint32_t half) const {
    const uint32_t counter[4] = {half, stream * 65536u + round, static_cast<uint32_t>(t),
                                 static_cast<uint32_t>(t >> 32)};
    const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
    uint32_t out[4];
    philox4x32_10(counter, key, out);
    return out[0] & ((uint32_t{1} << half_bits) - 1u);
  }

  uint64_t network(uint64_t v) const {
    const uint32_t half_mask = (uint32_t{1} << half_bits) - 1u;
    uint32_t left = static_cast<uint32_t>(v >> half_bits) & half_mask;
    uint32_t right = static_cast<uint32_t>(v) & half_mask;
    for (int round = 0; round < kFeistelRounds; ++round) {
      const uint32_t new_right = left ^ round_function(static_cast<uint32_t>(round), right);
      left = right;
      right = new_right;
    }
    return (static_cast<uint64_t>(left) << half_bits) | right;
  }

  uint64_t network_inverse(uint64_t v) const {
    const uint32_t half_mask = (uint32_t{1} << half_bits) - 1u;
    uint32_t left = static_cast<uint32_t>(v >> half_bits) & half_mask;
    uint32_t right = static_cast<uint32_t>(v) & half_mask;
    for (int round = kFeistelRounds - 1; round >= 0; --round) {
      const uint32_t old_left = right ^ round_function(static_cast<uint32_t>(round), left);
      right = left;
      left = old_left;
    }
    return (static_cast<uint64_t>(left) << half_bits) | right;
  }

  uint64_t forward(uint64_t v) const {
    do { v = network(v); } while (v >= B);
    return v;
  }
  uint64_t inverse(uint64_t v) const {
    do { v = network_inverse(v); } while (v >= B);
    return v;
  }
};

uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// number of blocks kept by a GRBS compressor of ratio R over B blocks (Definition 2 keeps B / R
// of them); non-integer quotients round up, R = 0 stands for the delta = 0 compressor C(v) = 0.
uint64_t blocks_kept(uint64_t B, uint64_t R) { return R == 0 ? 0 : ceil_div(B, R); }

void select_blocks(uint64_t seed, uint32_t stream, uint64_t t, uint64_t B, uint64_t k,
                   uint32_t* idx, uint8_t* mask) {
  BlockPermutation pi(seed, stream, t, B);
  for (uint64_t b = 0; b < B; ++b) mask[b] = 0;
  for (uint64_t j = 0; j < k; ++j) {
    const uint64_t b = pi.forward(j);
    if (idx) idx[j] = static_cast<uint32_t>(b);
    mask[b] = 1;
  }
}

// ---------------------------------------------------------------------------------
// The method.  All state arrays are [W][ld] row-major and hold the global columns
// [col0, col0 + ncols) of every worker's d-vector (col0 is a multiple of the block size).
// ---------------------------------------------------------------------------------
struct Problem {
  uint64_t d;        // parameters per worker
  uint32_t W;        // workers n
  uint32_t block;    // elements per GRBS block; B = ceil(d / block)
  uint64_t seed;     // the synchronized random seed
  uint64_t col0;     // first global column held by the arrays
  uint64_t ncols;    // number of columns held
  uint64_t ld;       // row stride of the arrays
  uint64_t num_blocks() const { return ceil_div(d, block); }
};

inline float fused_mul_add(float a, float b, float c) { return std::fmaf(a, b, c); }
inline double fused_mul_add(double a, double b, double c) { return std::fma(a, b, c); }

// GRBS, Definition 2: C(v) keeps v on the chosen blocks and is zero elsewhere.
template <class real>
void grbs_compress(const Problem& pb, const std::vector<uint8_t>& chosen, const real* v, real* cv) {
  for (uint64_t j = 0; j < pb.ncols; ++j) {
    const uint64_t b = (pb.col0 + j) / pb.block;
    cv[j] = chosen[b] ? v[j] : real(0);
  }
}

// PSync(v_i, C):  v'_i = C(v_i);  r_i = v_i - v'_i;  vbar' = (1/n) sum_i v'_i;  v'_i = vbar' + r_i.
// v, vprime, r are [W][ncols] dense temporaries.
template <class real>
void psync(const Problem& pb, const std::vector<uint8_t>& chosen, const std::vector<real>& v,
           std::vector<real>& vprime, std::vector<real>& r) {
  const uint64_t n = pb.ncols;
  for (uint32_t i = 0; i < pb.W; ++i) {
    grbs_compress(pb, chosen, &v[i * n], &vprime[i * n]);
    for (uint64_t j = 0; j < n; ++j) r[i * n + j] = v[i * n + j] - vprime[i * n + j];
  }
  std::vector<real> vbar(n);
  for (uint64_t j = 0; j < n; ++j) {
    real sum = vprime[j];
    for (uint32_t i = 1; i < pb.W; ++i) sum = sum + vprime[i * n + j];
    vbar[j] = sum / real(pb.W);
  }
  for (uint32_t i = 0; i < pb.W; ++i)
    for (uint64_t j = 0; j < n; ++j) vprime[i * n + j] = vbar[j] + r[i * n + j];
}

// Get_p with momentum:  m <- beta m + g;  p <- eta (beta m + g).   (Algorithm 3, the two
// statements after the gradient; Appendix A.4 Get_p.)  m is updated in place, p is [W][ncols].
template <class real>
void get_p(const Problem& pb, real eta, real beta, real* m, const real* g, std::vector<real>& p) {
  const uint64_t n = pb.ncols;
  for (uint32_t i = 0; i < pb.W; ++i)
    for (uint64_t j = 0; j < n; ++j) {
      real& mij = m[i * pb.ld + j];
      const real gij = g[i * pb.ld + j];
      mij = fused_mul_add(beta, mij, gij);
      p[i * n + j] = eta * fused_mul_add(beta, mij, gij);
    }
}

// Algorithm 3, iteration t, up to and including x_{t-1/2}, e_{t-1/2}:
//   p', r <- PSync(p, C_step);  x <- x - p';  e <- e - r.
template <class real>
void mcser_local_step(const Problem& pb, uint64_t t, uint64_t R_step, real eta, real beta, real* x,
                      real* e, real* m, const real* g) {
  const uint64_t n = pb.ncols, B = pb.num_blocks();
  std::vector<uint8_t> chosen(B);
  select_blocks(pb.seed, 0, t, B, blocks_kept(B, R_step), nullptr, chosen.data());
  std::vector<real> p(pb.W * n), pprime(pb.W * n), r(pb.W * n);
  get_p(pb, eta, beta, m, g, p);
  psync(pb, chosen, p, pprime, r);
  for (uint32_t i = 0; i < pb.W; ++i)
    for (uint64_t j = 0; j < n; ++j) {
      x[i * pb.ld + j] = x[i * pb.ld + j] - pprime[i * n + j];
      e[i * pb.ld + j] = e[i * pb.ld + j] - r[i * n + j];
    }
}

// Algorithm 3, the error-reset branch (t mod H = 0):
//   e', e_new <- PSync(e_{t-1/2}, C_reset);  x <- x_{t-1/2} - e_{t-1/2} + e'.
template <class real>
void mcser_error_reset(const Problem& pb, uint64_t t, uint64_t R_reset, real* x, real* e) {
  const uint64_t n = pb.ncols, B = pb.num_blocks();
  std::vector<uint8_t> chosen(B);
  select_blocks(pb.seed, 1, t, B, blocks_kept(B, R_reset), nullptr, chosen.data());
  std::vector<real> ehalf(pb.W * n), eprime(pb.W * n), r(pb.W * n);
  for (uint32_t i = 0; i < pb.W; ++i)
    for (uint64_t j = 0; j < n; ++j) ehalf[i * n + j] = e[i * pb.ld + j];
  psync(pb, chosen, ehalf, eprime, r);
  for (uint32_t i = 0; i < pb.W; ++i)
    for (uint64_t j = 0; j < n; ++j) {
      // Outside the chosen blocks C(e) = 0 on every worker, so e' = 0 + r = e exactly and the
      // correction -e + e' is identically zero: x is left as it is there.  (Evaluating (x - e) + e
      // in floating point would perturb x by a rounding on blocks the reset does not concern.)
      if (chosen[(pb.col0 + j) / pb.block])
        x[i * pb.ld + j] = (x[i * pb.ld + j] - ehalf[i * n + j]) + eprime[i * n + j];
      e[i * pb.ld + j] = r[i * n + j];
    }
}

// Implementation II (Appendix A.4): no residual buffer.
//   p', _ <- PSync(p, C_step);  x <- x - p'.
template <class real>
void cser2_local_step(const Problem& pb, uint64_t t, uint64_t R_step, real eta, real beta, real* x,
                      real* m, const real* g) {
  const uint64_t n = pb.ncols, B = pb.num_blocks();
  std::vector<uint8_t> chosen(B);
  select_blocks(pb.seed, 0, t, B, blocks_kept(B, R_step), nullptr, chosen.data());
  std::vector<real> p(pb.W * n), pprime(pb.W * n), r(pb.W * n);
  get_p(pb, eta, beta, m, g, p);
  psync(pb, chosen, p, pprime, r);
  for (uint32_t i = 0; i < pb.W; ++i)
    for (uint64_t j = 0; j < n; ++j) x[i * pb.ld + j] = x[i * pb.ld + j] - pprime[i * n + j];
}

//   x, _ <- PSync(x_{t-1/2}, C_reset)      (t mod H = 0)
template <class real>
void cser2_model_sync(const Problem& pb, uint64_t t, uint64_t R_reset, real* x) {
  const uint64_t n = pb.ncols, B = pb.num_blocks();
  std::vector<uint8_t> chosen(B);
  select_blocks(pb.seed, 1, t, B, blocks_kept(B, R_reset), nullptr, chosen.data());
  std::vector<real> xhalf(pb.W * n), xprime(pb.W * n), r(pb.W * n);
  for (uint32_t i = 0; i < pb.W; ++i)
    for (uint64_t j = 0; j < n; ++j) xhalf[i * n + j] = x[i * pb.ld + j];
  psync(pb, chosen, xhalf, xprime, r);
  for (uint32_t i = 0; i < pb.W; ++i)
    for (uint64_t j = 0; j < n; ++j) x[i * pb.ld + j] = xprime[i * n + j];
}

bool problem_ok(const Problem& pb) {
  return pb.d >= 1 && pb.W >= 1 && pb.block >= 1 && pb.ld >= pb.ncols &&
         pb.col0 % pb.block == 0 && pb.col0 + pb.ncols <= pb.d &&
         pb.num_blocks() <= 0xFFFFFFFFull;
}

}  // namespace

// ---------------------------------------------------------------------------------
// C entry points for the test-suite (ctypes).  Return 0 on success, -1 on a bad argument.
// ---------------------------------------------------------------------------------
extern "C" {

struct oracle_problem {
  uint64_t d;
  uint64_t seed;
  uint64_t col0;
  uint64_t ncols;
  uint64_t ld;
  uint32_t W;
  uint32_t block;
};

static Problem to_problem(const oracle_problem* q) {
  Problem pb;
  pb.d = q->d; pb.W = q->W; pb.block = q->block; pb.seed = q->seed;
  pb.col0 = q->col0; pb.ncols = q->ncols; pb.ld = q->ld;
  return pb;
}

void oracle_philox4x32_10(const uint32_t* counter, const uint32_t* key, uint32_t* out) {
  philox4x32_10(counter, key, out);
}

uint64_t oracle_blocks_kept(uint64_t B, uint64_t R) { return blocks_kept(B, R); }

uint64_t oracle_block_perm(uint64_t seed, uint32_t stream, uint64_t t, uint64_t B, uint64_t v) {
  return BlockPermutation(seed, stream, t, B).forward(v);
}

uint64_t oracle_block_perm_inverse(uint64_t seed, uint32_t stream, uint64_t t, uint64_t B,
                                   uint64_t v) {
  return BlockPermutation(seed, stream, t, B).inverse(v);
}

// idx: k entries in draw order (may be null); mask: B bytes.
int oracle_select_blocks(uint64_t seed, uint32_t stream, uint64_t t, uint64_t B, uint64_t k,
                         uint32_t* idx, uint8_t* mask) {
  if (B < 1 || B > 0xFFFFFFFFull || k > B || !mask) return -1;
  select_blocks(seed, stream, t, B, k, idx, mask);
  return 0;
}

#define ORACLE_INSTANTIATE(SUFFIX, REAL)                                                           \
  int oracle_mcser_local_step_##SUFFIX(const oracle_problem* q, uint64_t t, uint64_t R_step,       \
                                       double eta, double beta, REAL* x, REAL* e, REAL* m,         \
                                       const REAL* g) {                                            \
    const Problem pb = to_problem(q);                                                              \
    if (!problem_ok(pb) || !x || !e || !m || !g) return -1;                                        \
    mcser_local_step<REAL>(pb, t, R_step, REAL(eta), REAL(beta), x, e, m, g);                      \
    return 0;                                                                                      \
  }                                                                                                \
  int oracle_mcser_error_reset_##SUFFIX(const oracle_problem* q, uint64_t t, uint64_t R_reset,     \
                                        REAL* x, REAL* e) {                                        \
    const Problem pb = to_problem(q);                                                              \
    if (!problem_ok(pb) || !x || !e) return -1;                                                    \
    mcser_error_reset<REAL>(pb, t, R_reset, x, e);                                                 \
    return 0;                                                                                      \
  }                                                                                                \
  int oracle_cser2_local_step_##SUFFIX(const oracle_problem* q, uint64_t t, uint64_t R_step,       \
                                       double eta, double beta, REAL* x, REAL* m, const REAL* g) { \
    const Problem pb = to_problem(q);                                                              \
    if (!problem_ok(pb) || !x || !m || !g) return -1;                                              \
    cser2_local_step<REAL>(pb, t, R_step, REAL(eta), REAL(beta), x, m, g);                         \
    return 0;                                                                                      \
  }                                                                                                \
  int oracle_cser2_model_sync_##SUFFIX(const oracle_problem* q, uint64_t t, uint64_t R_reset,      \
                                       REAL* x) {                                                  \
    const Problem pb = to_problem(q);                                                              \
    if (!problem_ok(pb) || !x) return -1;                                                          \
    cser2_model_sync<REAL>(pb, t, R_reset, x);                                                     \
    return 0;                                                                                      \
  }

ORACLE_INSTANTIATE(f32, float)
ORACLE_INSTANTIATE(f64, double)

}  // extern "C"
