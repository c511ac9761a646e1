// Host part of the library: base-graph sampler, spectral test, mask object and
// the index expansions that need no GPU.
//
// Appendix "Ramanujan Bipartite Graph Generation": 2-lift, sparse biregular
// generation by log2(1/(1-sp)) lifts of a complete graph, rejection sampling
// until the graph meets the bound of Section 3.  Section 3: bipartite graph
// product = Kronecker product of biadjacency matrices.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <new>

#include "rbgp_internal.h"

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Fair coins for (seed, factor, attempt): counter-based SplitMix64.
struct Coins {
  uint64_t key, n = 0;
  Coins(uint64_t seed, uint64_t factor, uint64_t attempt)
      : key(mix64(mix64(mix64(seed) + factor) + attempt)) {}
  int next() {
    ++n;
    return int(mix64(key + n * kGolden) >> 63);
  }
};

using Bits = std::vector<uint8_t>;  // dense 0/1 matrix, row-major

// One random 2-lift: clone of u is u+a, clone of v is v+c; per edge (row-major
// order) coin 0 keeps the identity pair, coin 1 takes the crossover pair.
Bits lift2(const Bits &B, int a, int c, Coins &coins) {
  Bits L(size_t(4) * a * c, 0);
  const int c2 = 2 * c;
  for (int u = 0; u < a; ++u)
    for (int v = 0; v < c; ++v) {
      if (!B[size_t(u) * c + v]) continue;
      if (coins.next() == 0) {
        L[size_t(u) * c2 + v] = 1;
        L[size_t(u + a) * c2 + v + c] = 1;
      } else {
        L[size_t(u) * c2 + v + c] = 1;
        L[size_t(u + a) * c2 + v] = 1;
      }
    }
  return L;
}

Bits sample_biregular(int a, int c, int lifts, Coins &coins) {
  int ba = a >> lifts, bc = c >> lifts;
  Bits B(size_t(ba) * bc, 1);
  for (int l = 0; l < lifts; ++l) {
    B = lift2(B, ba, bc, coins);
    ba *= 2;
    bc *= 2;
  }
  return B;
}

// Eigenvalues of a symmetric n x n matrix by cyclic Jacobi rotations, descending.
std::vector<double> sym_eigenvalues(std::vector<double> A, int n) {
  auto at = [&](int i, int j) -> double & { return A[size_t(i) * n + j]; };
  double norm = 0;
  for (double x : A) norm += x * x;
  norm = std::sqrt(norm);
  for (int sweep = 0; sweep < 100; ++sweep) {
    double off = 0;
    for (int i = 0; i < n; ++i)
      for (int j = i + 1; j < n; ++j) off += at(i, j) * at(i, j);
    if (std::sqrt(2 * off) <= 1e-15 * norm || norm == 0) break;
    for (int p = 0; p < n; ++p)
      for (int q = p + 1; q < n; ++q) {
        double apq = at(p, q);
        if (std::fabs(apq) < 1e-300) continue;
        double theta = (at(q, q) - at(p, p)) / (2 * apq);
        double t = (theta >= 0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1));
        double cs = 1 / std::sqrt(t * t + 1), sn = t * cs;
        for (int k = 0; k < n; ++k) {
          double akp = at(k, p), akq = at(k, q);
          at(k, p) = cs * akp - sn * akq;
          at(k, q) = sn * akp + cs * akq;
        }
        for (int k = 0; k < n; ++k) {
          double apk = at(p, k), aqk = at(q, k);
          at(p, k) = cs * apk - sn * aqk;
          at(q, k) = sn * apk + cs * aqk;
        }
      }
  }
  std::vector<double> ev(n);
  for (int i = 0; i < n; ++i) ev[i] = at(i, i);
  std::sort(ev.begin(), ev.end(), [](double x, double y) { return x > y; });
  return ev;
}

// Largest eigenvalue of the symmetric tridiagonal matrix (diagonal al, off-diagonal be) by bisection
// on the number of eigenvalues above x (Sturm sequence of the leading principal minors).
double tridiagonal_top(const std::vector<double> &al, const std::vector<double> &be) {
  const int n = int(al.size());
  double lo = al[0], hi = al[0];
  for (int i = 0; i < n; ++i) {
    const double r = (i ? std::fabs(be[size_t(i) - 1]) : 0) + (i + 1 < n ? std::fabs(be[size_t(i)]) : 0);
    lo = std::min(lo, al[size_t(i)] - r);
    hi = std::max(hi, al[size_t(i)] + r);
  }
  auto above = [&](double x) {   // eigenvalues > x
    int count = 0;
    double q = 1;
    for (int i = 0; i < n; ++i) {
      const double b2 = i ? be[size_t(i) - 1] * be[size_t(i) - 1] : 0;
      q = al[size_t(i)] - x - (i ? b2 / q : 0);
      if (q == 0) q = 1e-300;
      if (q > 0) ++count;
    }
    return count;
  };
  for (int it = 0; it < 200 && hi - lo > 4e-16 * std::max(std::fabs(lo), std::fabs(hi)); ++it) {
    const double mid = 0.5 * (lo + hi);
    if (above(mid) >= 1) lo = mid; else hi = mid;
  }
  return 0.5 * (lo + hi);
}

// Second largest singular value of a large biregular graph.  Its largest one is sqrt(d_l d_r) with
// constant singular vectors, so the second is the largest singular value on the complement of the
// constant vector: Lanczos iteration on the smaller Gram operator restricted to that complement, with
// full reorthogonalisation, until the top Ritz value stands still.  Returns false when it has not
// converged within the step limit (the caller then takes the dense solver).
bool lanczos_sigma2(const Bits &B, int a, int c, double *s2) {
  const bool rows_small = a <= c;
  const int n = rows_small ? a : c, other = rows_small ? c : a;
  std::vector<std::vector<int>> nb_small(static_cast<size_t>(n)), nb_other(static_cast<size_t>(other));
  for (int u = 0; u < a; ++u)
    for (int v = 0; v < c; ++v)
      if (B[size_t(u) * c + v]) {
        nb_small[size_t(rows_small ? u : v)].push_back(rows_small ? v : u);
        nb_other[size_t(rows_small ? v : u)].push_back(rows_small ? u : v);
      }
  std::vector<double> mid(static_cast<size_t>(other));
  auto apply = [&](const std::vector<double> &x, std::vector<double> &y) {   // y = (Gram operator) x
    for (int o = 0; o < other; ++o) {
      double t = 0;
      for (int i : nb_other[size_t(o)]) t += x[size_t(i)];
      mid[size_t(o)] = t;
    }
    for (int i = 0; i < n; ++i) {
      double t = 0;
      for (int o : nb_small[size_t(i)]) t += mid[size_t(o)];
      y[size_t(i)] = t;
    }
  };
  auto deflate = [&](std::vector<double> &x) {   // remove the constant component
    double mean = 0;
    for (double t : x) mean += t;
    mean /= n;
    for (double &t : x) t -= mean;
  };
  const int max_steps = std::min(n - 1, 600);
  std::vector<std::vector<double>> Q;
  std::vector<double> al, be, q(static_cast<size_t>(n)), w(static_cast<size_t>(n));
  uint64_t state = 0x243F6A8885A308D3ull;   // fixed start vector
  for (double &t : q) {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    t = double(state >> 11) / double(1ull << 53) - 0.5;
  }
  deflate(q);
  double nrm = 0;
  for (double t : q) nrm += t * t;
  nrm = std::sqrt(nrm);
  for (double &t : q) t /= nrm;
  double previous = -1;
  for (int step = 0; step < max_steps; ++step) {
    Q.push_back(q);
    apply(q, w);
    double alpha = 0;
    for (int i = 0; i < n; ++i) alpha += w[size_t(i)] * q[size_t(i)];
    al.push_back(alpha);
    for (int pass = 0; pass < 2; ++pass) {   // orthogonal to everything so far, and to the constants
      for (const std::vector<double> &p : Q) {
        double dot = 0;
        for (int i = 0; i < n; ++i) dot += w[size_t(i)] * p[size_t(i)];
        for (int i = 0; i < n; ++i) w[size_t(i)] -= dot * p[size_t(i)];
      }
      deflate(w);
    }
    double beta = 0;
    for (double t : w) beta += t * t;
    beta = std::sqrt(beta);
    const bool exhausted = beta <= 1e-12 * std::max(1.0, std::fabs(alpha));   // invariant subspace
    if (exhausted || step % 10 == 9 || step + 1 == max_steps) {
      const double top = tridiagonal_top(al, be);
      if (exhausted || (previous >= 0 && std::fabs(top - previous) <= 1e-13 * std::max(top, 1.0))) {
        *s2 = std::sqrt(std::max(0.0, top));
        return true;
      }
      previous = top;
    }
    if (exhausted) break;
    be.push_back(beta);
    for (int i = 0; i < n; ++i) q[size_t(i)] = w[size_t(i)] / beta;
  }
  return false;
}

// Two largest singular values of the a x c 0/1 matrix B (eigenvalues of the
// smaller Gram matrix).  lambda_2 of the bipartite graph equals sigma_2.
void top_singular_dense(const Bits &B, int a, int c, double *s1, double *s2) {
  const bool rows_small = a <= c;
  const int n = rows_small ? a : c;
  std::vector<double> G(size_t(n) * n, 0.0);
  for (int i = 0; i < n; ++i)
    for (int j = i; j < n; ++j) {
      int dot = 0;
      if (rows_small)
        for (int k = 0; k < c; ++k) dot += B[size_t(i) * c + k] & B[size_t(j) * c + k];
      else
        for (int k = 0; k < a; ++k) dot += B[size_t(k) * c + i] & B[size_t(k) * c + j];
      G[size_t(i) * n + j] = G[size_t(j) * n + i] = dot;
    }
  std::vector<double> ev = sym_eigenvalues(G, n);
  *s1 = std::sqrt(std::max(0.0, ev[0]));
  *s2 = n > 1 ? std::sqrt(std::max(0.0, ev[1])) : 0.0;
}

// The same for a biregular graph with degrees (d, e) whose Ramanujan bound is `bound`: small graphs
// take the dense solver; larger ones (the dense one costs O(n^3): minutes at a thousand vertices)
// the iteration above, unless it fails to converge or lands so close to the bound that its last
// digits would decide the test.
void top_singular(const Bits &B, int a, int c, int d, int e, double bound, double *s1, double *s2) {
  if (std::min(a, c) > 192) {
    double s = 0;
    if (lanczos_sigma2(B, a, c, &s) && std::fabs(s - bound) > 1e-6 * bound) {
      *s1 = std::sqrt(double(d) * e);
      *s2 = s;
      return;
    }
  }
  top_singular_dense(B, a, c, s1, s2);
}

int ilog2_exact(int q) {  // log2(q) if q is a power of two, else -1
  if (q <= 0 || (q & (q - 1))) return -1;
  int l = 0;
  while ((1 << l) < q) ++l;
  return l;
}

thread_local char g_hip_error[256] = "";

}  // namespace

uint64_t rbgp_next_uid() {
  static std::atomic<uint64_t> next{1};
  return next.fetch_add(1);
}

void rbgp_set_hip_error(const char *msg) {
  std::strncpy(g_hip_error, msg ? msg : "", sizeof(g_hip_error) - 1);
  g_hip_error[sizeof(g_hip_error) - 1] = 0;
}

// Decide whether the MFMA kernels cover this mask and derive their tile shape.
// They need the RBGP4 roles: G_r and G_b complete (Section 5).
void rbgp_plan_mfma(rbgp_mask *m) {
  rbgp_mfma_plan p;
  const bool roles = m->d[1] == m->c[1] && m->d[3] == m->c[3];
  p.R = m->a[1] * m->a[3];
  p.RB = (p.R + 3) / 4;
  p.KS = m->d[2] * m->c[3];
  p.NCH = (p.KS + 15) / 16;
  p.SR = m->c[2] * m->c[3];
  p.packed_elems = int64_t(m->a[0]) * m->d[0] * m->c[1] * m->a[2] * p.RB * p.NCH * 64;
  p.ok = roles;
  m->plan = p;
}

// Register-streaming family: a stage is VC columns of G_r of one nonzero tile;
// its contraction list (v_r, j_i, v_b) has KCR <= 72 entries, padded to a stage size the
// kernels are built for.
void rbgp_plan_reg(rbgp_mask *m) {
  rbgp_reg_plan p;
  const bool roles = m->d[1] == m->c[1] && m->d[3] == m->c[3];
  p.A2 = m->a[1];
  while (p.A2 > 1 && p.A2 * m->a[3] > 16) {   // largest divisor of |G_r.U| that fits the MFMA group
    --p.A2;
    while (m->a[1] % p.A2) --p.A2;
  }
  p.fold = m->a[1] / p.A2;
  p.TR = m->a[0] * p.fold;
  p.R = p.A2 * m->a[3];
  p.RB = (p.R + 3) / 4;
  p.KT = m->c[1] * m->d[2] * m->c[3];
  const int per_v = m->d[2] * m->c[3];
  p.VC = 0;
  for (int vc = m->c[1]; vc >= 1; --vc)
    if (m->c[1] % vc == 0 && vc * per_v <= 72) { p.VC = vc; break; }
  p.ok = roles && p.VC > 0 && p.R <= 16;   // (R > 16 only when |G_b.U| alone exceeds 16)
  if (p.ok) {
    p.KCR = p.VC * per_v;
    p.KC = p.KCR <= 8 ? 8 : p.KCR <= 18 ? 18 : p.KCR <= 32 ? 32 : p.KCR <= 36 ? 36 : 72;
    p.NSTG = m->c[1] / p.VC;
    p.SRC = p.VC * m->c[2] * m->c[3];
    p.RS = 2;
    while (p.RS < p.R) p.RS *= 2;
    p.MG = 16 / p.RS;
    p.NO = (p.KC + 3) / 4;
    p.NQ = (p.NO + 3) / 4;
    // one more all-zero fragment ends the buffer
    p.packed_elems = (int64_t(p.TR) * m->d[0] * p.NSTG * m->a[2] + 1) * p.NQ * 4 * p.RS * 4;
    const int nq_bf16 = rbgp_bf16_blocks32(p.KC) + (rbgp_bf16_tail16(p.KC) ? 1 : 0);
    p.packed_elems_bf16 = (int64_t(p.TR) * m->d[0] * p.NSTG * m->a[2] + 1) * nq_bf16 * 4 * p.RS * 8;
  }
  m->reg = p;
  if (p.ok) rbgp_reg_cluster(m, p.MG, &m->reg_clusters);
  rbgp_reg_plan_dual(m, &m->reg_dual);
}

// The mask with G_i filled in, for RBGP_KERNEL_MFMA_REG_FILLED.  G_r (x) G_i with both complete is the complete
// graph on their vertices, so the filled mask is G_o (x) J(a_r a_i, c_r c_i) (x) J(1, 1) (x) G_b: a four-factor mask
// of the same family with the same row and column numbering (Kronecker ordering), every kept position of this
// mask among its own.  Its a_r a_i a_b rows per tile row share one column set, which is what the 16-row MFMA
// groups of the register family want; the price is a zero stored and multiplied wherever G_i has no edge.
// Built only where that can pay: few rows per column set here (<= 4), a sparse G_i, and a filled mask the
// register family covers.
// A second way to the same end, where G_o is at least a quarter full: G_o filled in.  The filled G_o is complete, so
// G_o (x) G_r merges into one tile column (see rbgp_plan_regroup) and the stages become runs of up to 72 steps
// through all of K instead of the few steps one tile holds; every tile row has that one tile, so groups of several
// tile rows are full.  c_o / d_o times the products.  Of the two candidates the one whose walk is cheaper (per stage
// ~110 cycles + 36 per padded step) is kept; AUTO then weighs it against the mask as given.
static rbgp_mask *filled_twin(const rbgp_mask *m, int kind) {
  const bool roles = m->d[1] == m->c[1] && m->d[3] == m->c[3];
  if (!roles || (m->c[3] == 9 && m->d[3] == 9 && kind == 1)) return nullptr;
  int32_t a[4], c[4], d[4];
  int64_t rowdeg, coldeg;
  if (kind == 0) {
    if (m->d[2] == m->c[2] || int64_t(m->a[1]) * m->a[3] > 4) return nullptr;
    const int64_t ar = int64_t(m->a[1]) * m->a[2], cr = int64_t(m->c[1]) * m->c[2];
    if (ar > (1 << 20) || cr > (1 << 20)) return nullptr;
    const int32_t aa[4] = {m->a[0], int32_t(ar), 1, m->a[3]}, cc[4] = {m->c[0], int32_t(cr), 1, m->c[3]};
    for (int i = 0; i < 4; ++i) { a[i] = aa[i]; c[i] = cc[i]; d[i] = i == 0 ? m->d[0] : cc[i]; }
    rowdeg = int64_t(m->d[0]) * cr * m->c[3];
    coldeg = int64_t(m->e[0]) * ar * m->a[3];
  } else {
    if (m->d[0] == m->c[0] || int64_t(m->c[0]) > 4 * int64_t(m->d[0])) return nullptr;
    const int64_t cr = int64_t(m->c[0]) * m->c[1];
    if (cr > (1 << 20)) return nullptr;
    // (both G_o and G_r complete now: their rows merge as well, J(a_o, 1) (x) J(a_r, c_o c_r) = J(1, 1) (x) J(a_o a_r, c_o c_r),
    // so all a_o a_r |G_b.U| rows of a G_i vertex share one column set: full MFMA groups whatever |G_r.U| |G_b.U| is)
    const int64_t ar = int64_t(m->a[0]) * m->a[1];
    if (ar > (1 << 20)) return nullptr;
    const int32_t aa[4] = {1, int32_t(ar), m->a[2], m->a[3]}, cc[4] = {1, int32_t(cr), m->c[2], m->c[3]};
    for (int i = 0; i < 4; ++i) { a[i] = aa[i]; c[i] = cc[i]; d[i] = i == 2 ? m->d[2] : cc[i]; }
    rowdeg = cr * m->d[2] * m->c[3];
    coldeg = ar * m->e[2] * m->a[3];
  }
  if (m->M * rowdeg >= (int64_t(1) << 31)) return nullptr;
  rbgp_mask *t = new rbgp_mask();
  try {
    for (int i = 0; i < 4; ++i) {
      const bool same = kind == 0 ? i == 0 : i == 2;     // the factor the twin shares with the mask
      t->a[i] = a[i]; t->c[i] = c[i]; t->d[i] = d[i];
      t->e[i] = same ? m->e[i] : a[i];
      t->sigma1[i] = same ? m->sigma1[i] : std::sqrt(double(a[i]) * c[i]);
      t->sigma2[i] = same ? m->sigma2[i] : 0.0;
      t->bound[i] = same ? m->bound[i] : std::sqrt(double(t->d[i] - 1)) + std::sqrt(double(t->e[i] - 1));
      t->status[i] = same ? m->status[i] : RBGP_SPEC_COMPLETE;
      t->tries[i] = 0;
      if (same) {
        t->adj[i] = m->adj[i];
      } else {
        t->adj[i].resize(size_t(a[i]) * c[i]);
        for (int u = 0; u < a[i]; ++u)
          for (int v = 0; v < c[i]; ++v) t->adj[i][size_t(u) * c[i] + v] = v;
      }
    }
    t->M = m->M; t->K = m->K; t->rowdeg = rowdeg; t->coldeg = coldeg; t->nnz = m->M * rowdeg;
    t->kernel_choice = RBGP_KERNEL_MFMA_REG;
    t->uid = rbgp_next_uid();
    t->dev = nullptr;
    rbgp_plan_mfma(t);
    rbgp_plan_reg(t);
    if (!rbgp_reg_covers(t) || t->reg.packed_elems * 4 > (int64_t(1) << 30)) {
      delete t;
      return nullptr;
    }
  } catch (...) {
    delete t;
    throw;
  }
  return t;
}

void rbgp_plan_filled(rbgp_mask *m) {
  m->filled = nullptr;
  m->filled_kind = 0;
  auto walk_cost = [](const rbgp_mask *x) {
    int64_t n = 0;
    for (int32_t c : x->reg_clusters.counts) n += c;
    return n * (110 + 36 * x->reg.KC) * x->a[2];
  };
  rbgp_mask *t0 = filled_twin(m, 0), *t1 = nullptr;
  try {
    t1 = filled_twin(m, 1);
  } catch (...) {
    delete t0;
    throw;
  }
  if (t0 && t1) {
    if (walk_cost(t1) < walk_cost(t0)) { delete t0; t0 = nullptr; } else { delete t1; t1 = nullptr; }
  }
  m->filled = t0 ? t0 : t1;
  m->filled_kind = t0 ? 0 : 1;
}

// The same mask with part of G_b's rows moved into G_i, for RBGP_KERNEL_MFMA_REG.  Where more than 16 rows share a
// column set (|G_r.U| |G_b.U| > 16), the plan moves rows of G_r into the tile-row index until the rest fits a 16-row
// MFMA group; with |G_b.U| = 9 (the transpose of a lowered 3x3 convolution) that leaves 9 rows of 16.  A complete
// G_b is a Kronecker product itself, J(a_b, c_b) = J(q, 1) (x) J(a_b / q, c_b), and G_i (x) J(q, 1) is a biregular
// graph again (every vertex of G_i repeated q times), so
//   G_o (x) G_r (x) G_i (x) G_b = G_o (x) G_r (x) (G_i (x) J(q, 1)) (x) J(a_b / q, c_b)
// entry for entry, with the same numbering of rows and columns and the same order of a row's kept values: another
// four-factor mask of the family, with |G_r.U| a_b / q rows per column set.  The q that fills the MFMA group best is
// taken (9 = 3 x 3: 12 rows of 16 with |G_r.U| = 4 instead of 9), if it beats the plan of the mask as given.  Not
// for the mask of a lowered 3x3 convolution itself (rbgp_conv3x3 reads that mask's own layout).
//
// The column side has the same freedom where G_o is complete: J(a_o, c_o) (x) J(a_r, c_r) = J(a_o, 1) (x) J(a_r, c_o c_r),
// one tile column that holds all of K.  A stage is a run of columns of G_r inside a tile, so with few columns in G_r
// the stages are short however dense the mask (Table 2's cells with a complete G_o: |G_r.V| = 1, stages of 2 to 8
// steps padded to 8, 128 of them per wave); on the merged factoring they are 64 steps of 72.  Both dtypes.
static bool plan_regroup_columns(rbgp_mask *m);

void rbgp_plan_regroup(rbgp_mask *m) {
  m->regroup = nullptr;
  m->regroup_bf16 = false;
  const rbgp_reg_plan &p = m->reg;
  if (!p.ok || !rbgp_reg_covers(m)) return;
  if ((m->c[3] == 9 && m->d[3] == 9) || m->d[3] != m->c[3] || m->d[1] != m->c[1]) return;
  if (plan_regroup_columns(m)) return;
  if (p.fold <= 1) return;
  for (int u = 0; u < m->a[3]; ++u)      // (a complete G_b lists its columns in order: the canonical order carries over)
    for (int v = 0; v < m->c[3]; ++v)
      if (m->adj[3][size_t(u) * m->c[3] + v] != v) return;
  int best_rows = 0, best_r = p.R;
  for (int rows = 1; rows < m->a[3]; ++rows) {   // rows of G_b kept in the last factor
    if (m->a[3] % rows) continue;
    int a2 = m->a[1];                            // what the plan would leave of G_r (see rbgp_plan_reg)
    while (a2 > 1 && a2 * rows > 16) {
      --a2;
      while (m->a[1] % a2) --a2;
    }
    if (a2 * rows <= 16 && a2 * rows >= best_r + (best_rows ? 0 : 1)) {
      best_r = a2 * rows;
      best_rows = rows;
    }
  }
  if (!best_rows) return;
  const int q = m->a[3] / best_rows;
  if (int64_t(m->a[2]) * q > (1 << 20)) return;
  rbgp_mask *t = new rbgp_mask();
  try {
    for (int i = 0; i < 4; ++i) {
      t->a[i] = m->a[i]; t->c[i] = m->c[i]; t->d[i] = m->d[i]; t->e[i] = m->e[i];
      t->sigma1[i] = m->sigma1[i]; t->sigma2[i] = m->sigma2[i]; t->bound[i] = m->bound[i];
      t->status[i] = m->status[i]; t->tries[i] = 0;
      t->adj[i] = m->adj[i];
    }
    t->a[2] = m->a[2] * q; t->e[2] = m->e[2] * q;
    t->sigma1[2] = m->sigma1[2] * std::sqrt(double(q)); t->sigma2[2] = m->sigma2[2] * std::sqrt(double(q));
    t->a[3] = best_rows; t->e[3] = best_rows;
    t->sigma1[3] = std::sqrt(double(best_rows) * m->c[3]);
    t->adj[2].resize(size_t(t->a[2]) * m->d[2]);
    for (int u = 0; u < m->a[2]; ++u)
      for (int b = 0; b < q; ++b)
        for (int j = 0; j < m->d[2]; ++j)
          t->adj[2][(size_t(u) * q + b) * m->d[2] + j] = m->adj[2][size_t(u) * m->d[2] + j];
    t->adj[3].resize(size_t(best_rows) * m->c[3]);
    for (int u = 0; u < best_rows; ++u)
      for (int v = 0; v < m->c[3]; ++v) t->adj[3][size_t(u) * m->c[3] + v] = v;
    t->M = m->M; t->K = m->K; t->rowdeg = m->rowdeg; t->coldeg = m->coldeg; t->nnz = m->nnz;
    t->kernel_choice = RBGP_KERNEL_MFMA_REG;
    t->uid = rbgp_next_uid();
    t->dev = nullptr;
    rbgp_plan_mfma(t);
    rbgp_plan_reg(t);
    if (!rbgp_reg_covers(t) || t->reg.R <= p.R) {
      delete t;
      return;
    }
  } catch (...) {
    delete t;
    throw;
  }
  m->regroup = t;
}

static bool plan_regroup_columns(rbgp_mask *m) {
  const rbgp_reg_plan &p = m->reg;
  if (m->c[0] <= 1 || m->d[0] != m->c[0] || p.KC >= 72) return false;
  if (int64_t(m->c[0]) * m->c[1] > (1 << 20) || int64_t(m->a[0]) * m->a[1] > (1 << 20)) return false;
  for (int i = 0; i < 2; ++i)     // (complete factors that list their columns in order: the canonical order carries over)
    for (int u = 0; u < m->a[i]; ++u)
      for (int v = 0; v < m->c[i]; ++v)
        if (m->adj[i][size_t(u) * m->c[i] + v] != v) return false;
  rbgp_mask *t = new rbgp_mask();
  try {
    for (int i = 0; i < 4; ++i) {
      t->a[i] = m->a[i]; t->c[i] = m->c[i]; t->d[i] = m->d[i]; t->e[i] = m->e[i];
      t->sigma1[i] = m->sigma1[i]; t->sigma2[i] = m->sigma2[i]; t->bound[i] = m->bound[i];
      t->status[i] = m->status[i]; t->tries[i] = 0;
      t->adj[i] = m->adj[i];
    }
    const int cr = m->c[0] * m->c[1];
    // (the rows merge too: J(a_o, 1) (x) J(a_r, c_o c_r) = J(1, 1) (x) J(a_o a_r, c_o c_r), more rows per column set)
    const int ar = m->a[0] * m->a[1];
    t->a[0] = 1; t->c[0] = 1; t->d[0] = 1; t->e[0] = 1; t->sigma1[0] = 1.0; t->sigma2[0] = 0.0;
    t->a[1] = ar; t->c[1] = cr; t->d[1] = cr; t->e[1] = ar; t->sigma1[1] = std::sqrt(double(ar) * cr); t->sigma2[1] = 0.0;
    t->adj[0].assign(1, 0);
    t->adj[1].resize(size_t(ar) * cr);
    for (int u = 0; u < ar; ++u)
      for (int v = 0; v < cr; ++v) t->adj[1][size_t(u) * cr + v] = v;
    t->M = m->M; t->K = m->K; t->rowdeg = m->rowdeg; t->coldeg = m->coldeg; t->nnz = m->nnz;
    t->kernel_choice = RBGP_KERNEL_MFMA_REG;
    t->uid = rbgp_next_uid();
    t->dev = nullptr;
    rbgp_plan_mfma(t);
    rbgp_plan_reg(t);
    // taken where the stages get longer and the walk cheaper (per stage ~110 cycles + 36 per padded step, the fp32
    // kernels' measured cost; bf16 follows the same order)
    auto walk_cost = [](const rbgp_mask *x) {
      int64_t n = 0;
      for (int32_t c : x->reg_clusters.counts) n += c;
      return n * (110 + 36 * x->reg.KC) * x->a[2];
    };
    if (!rbgp_reg_covers(t) || t->reg.KC <= p.KC || walk_cost(t) >= walk_cost(m)) {
      delete t;
      return false;
    }
  } catch (...) {
    delete t;
    throw;
  }
  m->regroup = t;
  m->regroup_bf16 = true;
  return true;
}

// Register-streaming family: group the tile rows into clusters of U whose adjacency lists
// overlap most (greedy: seed with the lowest free tile row, add the free row that enlarges
// the union of tiles least; then local search, and exhaustive matching for pairs), and
// list for every cluster the stages it walks.
void rbgp_reg_cluster(const rbgp_mask *m, int U, rbgp_reg_clusters *out) {
  const rbgp_reg_plan &pl = m->reg;
  const int a1 = pl.TR, c1 = m->c[0], d1 = m->d[0];   // tile rows; tile row u has G_o's row u / fold
  const int ncl = (a1 + U - 1) / U;
  std::vector<int32_t> members(size_t(ncl) * U, -1);
  std::vector<char> used(a1, 0);
  std::vector<std::vector<char>> has(a1, std::vector<char>(c1, 0));
  for (int u = 0; u < a1; ++u)
    for (int j = 0; j < d1; ++j) has[u][m->adj[0][size_t(u / pl.fold) * d1 + j]] = 1;
  // The searches below cost about a1^2 * c1 (greedy) and ncl^2 * U^3 * c1 per pass (local search):
  // fine for the tile counts of a layer, not for base graphs of thousands of vertices, whose tile
  // rows share few tiles whatever the grouping; those keep consecutive tile rows together.
  const double greedy_cost = double(a1) * a1 * c1, search_cost = double(ncl) * ncl * U * U * U * c1;
  const bool cheap = greedy_cost <= 2e8;
  if (!cheap)
    for (int u = 0; u < a1; ++u) members[size_t(u)] = u;
  for (int c = 0; cheap && c < ncl; ++c) {
    std::vector<char> uni(c1, 0);
    for (int k = 0; k < U; ++k) {
      int best = -1, best_grow = 1 << 30;
      for (int u = 0; u < a1; ++u) {
        if (used[u]) continue;
        int grow = 0;
        for (int v = 0; v < c1; ++v) grow += has[u][v] && !uni[v];
        if (grow < best_grow) { best_grow = grow; best = u; }
      }
      if (best < 0) break;
      used[best] = 1;
      members[size_t(c) * U + k] = best;
      for (int v = 0; v < c1; ++v) uni[v] |= has[best][v];
    }
  }
  // Local search: swap members between two clusters while that lowers the larger of their
  // two unions, or keeps it and lowers the sum.  The longest cluster sets the kernel's
  // duration (one wave per SIMD), the sum its total work.
  auto union_size = [&](int c) {
    int n = 0;
    for (int v = 0; v < c1; ++v) {
      bool any = false;
      for (int k = 0; k < U; ++k) any |= members[size_t(c) * U + k] >= 0 && has[members[size_t(c) * U + k]][v];
      n += any;
    }
    return n;
  };
  for (bool improved = cheap && search_cost <= 2e8; improved;) {
    improved = false;
    for (int ca = 0; ca < ncl; ++ca)
      for (int cb = ca + 1; cb < ncl; ++cb)
        for (int ka = 0; ka < U; ++ka)
          for (int kb = 0; kb < U; ++kb) {
            const int ua = union_size(ca), ub = union_size(cb);
            std::swap(members[size_t(ca) * U + ka], members[size_t(cb) * U + kb]);
            const int na = union_size(ca), nb = union_size(cb);
            const bool better = std::max(na, nb) < std::max(ua, ub) ||
                                (std::max(na, nb) == std::max(ua, ub) && na + nb < ua + ub);
            if (better)
              improved = true;
            else
              std::swap(members[size_t(ca) * U + ka], members[size_t(cb) * U + kb]);
          }
  }
  // Pairs (U == 2): exhaustive matching by depth-first search with the local-search result
  // as the bound, minimising (largest union, sum of unions); bounded effort.
  if (U == 2 && a1 % 2 == 0 && a1 <= 64) {
    std::vector<std::vector<int>> un(a1, std::vector<int>(a1, 0));
    for (int x = 0; x < a1; ++x)
      for (int y = 0; y < a1; ++y) {
        int n = 0;
        for (int v = 0; v < c1; ++v) n += has[x][v] || has[y][v];
        un[x][y] = n;
      }
    int best_max = 0, best_sum = 0;
    for (int c = 0; c < ncl; ++c) {
      const int n = un[members[2 * c]][members[2 * c + 1]];
      best_max = std::max(best_max, n);
      best_sum += n;
    }
    std::vector<int32_t> cur(members.size()), best = members;
    std::vector<char> taken(a1, 0);
    long budget = 4000000;
    // recursive lambda via explicit std::function-free trick
    struct Rec {
      const std::vector<std::vector<int>> &un; std::vector<int32_t> &cur, &best; std::vector<char> &taken;
      int a1; int &best_max, &best_sum; long &budget;
      void go(int depth, int cmax, int csum) {
        if (budget-- <= 0) return;
        int x = 0;
        while (x < a1 && taken[x]) ++x;
        if (x == a1) {
          if (cmax < best_max || (cmax == best_max && csum < best_sum)) { best_max = cmax; best_sum = csum; best = cur; }
          return;
        }
        taken[x] = 1;
        for (int y = x + 1; y < a1; ++y) {
          if (taken[y]) continue;
          const int n = un[x][y], nmax = std::max(cmax, n), nsum = csum + n;
          if (nmax > best_max || (nmax == best_max && nsum >= best_sum)) continue;
          taken[y] = 1;
          cur[2 * depth] = x; cur[2 * depth + 1] = y;
          go(depth + 1, nmax, nsum);
          taken[y] = 0;
        }
        taken[x] = 0;
      }
    } rec{un, cur, best, taken, a1, best_max, best_sum, budget};
    rec.go(0, 0, 0);
    members = best;
  }
  std::vector<int32_t> counts(ncl, 0);
  int longest = 0;
  for (int c = 0; c < ncl; ++c) {
    int tiles = 0;
    for (int v1 = 0; v1 < c1; ++v1) {
      bool any = false;
      for (int k = 0; k < U; ++k) any |= members[size_t(c) * U + k] >= 0 && has[members[size_t(c) * U + k]][v1];
      tiles += any;
    }
    longest = std::max(longest, tiles * pl.NSTG);
  }
  const int TS = longest > kRegWaveStages ? 256 : 64;
  const int stored = TS;   // (entries past a list's end stay -1)
  std::vector<int32_t> stages(size_t(ncl) * (1 + U) * TS, -1);
  for (int c = 0; c < ncl; ++c) {
    int st = 0;
    for (int v1 = 0; v1 < c1; ++v1) {
      bool any = false;
      for (int k = 0; k < U; ++k) any |= members[size_t(c) * U + k] >= 0 && has[members[size_t(c) * U + k]][v1];
      if (!any) continue;
      for (int sg = 0; sg < pl.NSTG; ++sg, ++st) {
        if (st >= stored) continue;   // does not fit the table: counted, not stored
        stages[(size_t(c) * (1 + U)) * TS + st] =
            int32_t((int64_t(v1) * m->c[1] + int64_t(sg) * pl.VC) * m->c[2] * m->c[3]);
        for (int k = 0; k < U; ++k) {
          const int u1 = members[size_t(c) * U + k];
          if (u1 < 0 || !has[u1][v1]) continue;
          int j1 = 0;
          while (m->adj[0][size_t(u1 / pl.fold) * d1 + j1] != v1) ++j1;
          stages[(size_t(c) * (1 + U) + 1 + k) * TS + st] = j1 * pl.NSTG + sg;
        }
      }
    }
    counts[c] = st;
  }
  out->U = U;
  out->ncl = ncl;
  out->tstride = TS;
  out->max_stages = 0;
  for (int c = 0; c < ncl; ++c) out->max_stages = std::max(out->max_stages, int(counts[c]));
  out->members.swap(members);
  out->stages.swap(stages);
  out->counts.swap(counts);
}

// Register-streaming family, lo/hi pairing (see rbgp_reg_dual): choose the quads (L0, L1, H0, H1)
// and give every tile of an H row to a wave whose L row has the same tile.  The two waves of an L
// row share a SIMD, so a quad costs, per L row, the tiles of that row plus its share of the H tiles
// that no L row can carry; the search minimises (longest pair of waves, total) over the partitions of
// the tile rows into quads: depth first, candidates in order of cost, bounded effort.  Two rows with
// complementary tile sets (the two clones of a vertex after the last 2-lift of a complete graph,
// Appendix) make a perfect L pair for any such H pair: every stage then multiplies 16 rows of the mask.
void rbgp_reg_plan_dual(const rbgp_mask *m, rbgp_reg_dual *out) {
  *out = rbgp_reg_dual();
  const rbgp_reg_plan &pl = m->reg;
  if (!pl.ok || pl.MG != 2 || pl.TR < 2) return;
  const int TR = pl.TR, TRP = (TR + 3) / 4 * 4, c1 = m->c[0], d1 = m->d[0];
  if (TRP > 32 || c1 > 256) return;
  constexpr int W = 4;   // 64-bit words of a tile set
  struct Set { uint64_t w[W]; };
  std::vector<Set> has(static_cast<size_t>(TRP), Set{{0, 0, 0, 0}});
  for (int u = 0; u < TR; ++u)
    for (int j = 0; j < d1; ++j) {
      const int v = m->adj[0][size_t(u / pl.fold) * d1 + j];
      has[size_t(u)].w[v >> 6] |= uint64_t(1) << (v & 63);
    }
  auto tiles = [&](int u) { return u < TR ? d1 : 0; };
  // stages of the busier L row and of the whole quad for the ordered roles (L0, L1, H0, H1)
  auto cost = [&](int l0, int l1, int h0, int h1, int *total) {
    int extra = 0;
    for (int k = 0; k < W; ++k) {
      const uint64_t a = has[size_t(l0)].w[k], b = has[size_t(l1)].w[k], x = has[size_t(h0)].w[k], y = has[size_t(h1)].w[k];
      extra += __builtin_popcountll(x & ~(a | b)) + __builtin_popcountll(y & ~(a | b)) + __builtin_popcountll(x & y & (a ^ b));
    }
    const int t0 = tiles(l0), t1 = tiles(l1);
    *total = t0 + t1 + extra;
    return std::max(std::max(t0, t1), (*total + 1) / 2);
  };
  struct Cand { int mx, tot, r[4]; };
  const int nq = TRP / 4;
  std::vector<int32_t> cur(static_cast<size_t>(TRP), 0), best;
  int best_max = 1 << 30, best_tot = 1 << 30;
  std::vector<char> taken(static_cast<size_t>(TRP), 0);
  long budget = 200000;
  const int lb_tot = (TR * d1 + 1) / 2;
  struct Rec {
    decltype(cost) &quad_cost; std::vector<int32_t> &cur, &best; std::vector<char> &taken;
    int TRP, nq, d1, lb_tot; int &best_max, &best_tot; long &budget;
    bool done() const { return best_max <= d1 && best_tot <= lb_tot; }
    void go(int depth, int cmax, int ctot) {
      if (depth == nq) {
        if (cmax < best_max || (cmax == best_max && ctot < best_tot)) { best_max = cmax; best_tot = ctot; best = cur; }
        return;
      }
      int x = 0;
      while (taken[size_t(x)]) ++x;
      std::vector<Cand> cands;
      for (int y = x + 1; y < TRP; ++y) {
        if (taken[size_t(y)]) continue;
        for (int z = y + 1; z < TRP; ++z) {
          if (taken[size_t(z)]) continue;
          for (int w = z + 1; w < TRP; ++w) {
            if (taken[size_t(w)]) continue;
            const int q[4] = {x, y, z, w};
            // the six choices of the L pair
            for (int a = 0; a < 4; ++a)
              for (int b = a + 1; b < 4; ++b) {
                int h[2], nh = 0;
                for (int k = 0; k < 4; ++k)
                  if (k != a && k != b) h[nh++] = q[k];
                Cand c;
                c.mx = quad_cost(q[a], q[b], h[0], h[1], &c.tot);
                c.r[0] = q[a]; c.r[1] = q[b]; c.r[2] = h[0]; c.r[3] = h[1];
                cands.push_back(c);
              }
          }
        }
      }
      std::stable_sort(cands.begin(), cands.end(), [](const Cand &p, const Cand &q) {
        return p.mx != q.mx ? p.mx < q.mx : p.tot < q.tot;
      });
      for (const Cand &c : cands) {
        if (budget-- <= 0 || done()) return;
        const int nmax = std::max(cmax, c.mx), ntot = ctot + c.tot;
        if (nmax > best_max || (nmax == best_max && ntot >= best_tot)) continue;
        for (int k = 0; k < 4; ++k) { taken[size_t(c.r[k])] = 1; cur[size_t(4 * depth + k)] = c.r[k]; }
        go(depth + 1, nmax, ntot);
        for (int k = 0; k < 4; ++k) taken[size_t(c.r[k])] = 0;
      }
    }
  } rec{cost, cur, best, taken, TRP, nq, d1, lb_tot, best_max, best_tot, budget};
  rec.go(0, 0, 0);
  if (best.empty()) return;

  // Stage lists of the four waves (x, y) = (L_x, H_y) of every quad.
  auto has_tile = [&](int u, int v) { return u < TR && ((has[size_t(u)].w[v >> 6] >> (v & 63)) & 1); };
  auto pos = [&](int u, int v) {   // position of v in u's adjacency list
    int j = 0;
    while (m->adj[0][size_t(u / pl.fold) * d1 + j] != v) ++j;
    return j;
  };
  struct Stage { int v, lo, hi; };   // tile, position in L_x's list (-1: none), position in H_y's list (-1: none)
  out->members.assign(size_t(nq) * 4, -1);
  out->stages.assign(size_t(nq) * 4 * 3 * 64, -1);
  out->counts.assign(size_t(nq) * 4, 0);
  std::vector<std::vector<Stage>> lists(size_t(nq) * 4);
  for (int q = 0; q < nq; ++q) {
    const int L[2] = {best[size_t(4 * q)], best[size_t(4 * q + 1)]}, H[2] = {best[size_t(4 * q + 2)], best[size_t(4 * q + 3)]};
    for (int k = 0; k < 4; ++k) out->members[size_t(4 * q + k)] = best[size_t(4 * q + k)] < TR ? best[size_t(4 * q + k)] : -1;
    std::vector<Stage> st[2][2];
    std::vector<std::pair<int, int>> lo_only, hi_only;   // (tile, x) / (tile, y) without a partner
    for (int v = 0; v < c1; ++v) {
      int hs[2], nh = 0;
      for (int y = 0; y < 2; ++y)
        if (has_tile(H[y], v)) hs[nh++] = y;
      const bool l[2] = {has_tile(L[0], v), has_tile(L[1], v)};
      int used = 0;
      if (l[0] && l[1] && nh == 2) {
        st[0][0].push_back({v, pos(L[0], v), pos(H[0], v)});
        st[1][1].push_back({v, pos(L[1], v), pos(H[1], v)});
        used = 2;
      } else {
        for (int x = 0; x < 2; ++x) {
          if (!l[x]) continue;
          if (used < nh) {
            st[x][hs[used]].push_back({v, pos(L[x], v), pos(H[hs[used]], v)});
            ++used;
          } else {
            lo_only.push_back({v, x});
          }
        }
      }
      for (; used < nh; ++used) hi_only.push_back({v, hs[used]});
    }
    // a tile of L_x alone goes to the shorter of L_x's two waves; a tile of H_y alone to the L row
    // with fewer stages so far (the two waves of an L row share a SIMD)
    for (const auto &e : lo_only) {
      const int x = e.second, y = st[x][1].size() < st[x][0].size() ? 1 : 0;
      st[x][y].push_back({e.first, pos(L[x], e.first), -1});
    }
    for (const auto &e : hi_only) {
      const int y = e.second;
      const int x = st[1][0].size() + st[1][1].size() < st[0][0].size() + st[0][1].size() ? 1 : 0;
      st[x][y].push_back({e.first, -1, pos(H[y], e.first)});
    }
    for (int x = 0; x < 2; ++x)
      for (int y = 0; y < 2; ++y) lists[(size_t(q) * 2 + x) * 2 + y] = st[x][y];
  }
  for (int q = 0; q < nq; ++q) {
    for (int x = 0; x < 2; ++x) {
      int both = 0;
      for (int y = 0; y < 2; ++y) {
        std::vector<Stage> &l = lists[(size_t(q) * 2 + x) * 2 + y];
        // (ascending tiles; a common order of the tiles chosen so that the r-th tiles of all waves are few distinct
        // ones -- four waves read every tile, all in the same round -- measured no faster)
        std::stable_sort(l.begin(), l.end(), [](const Stage &a, const Stage &b) { return a.v < b.v; });
        int n = 0;
        int32_t *tab = &out->stages[((size_t(q) * 2 + x) * 2 + y) * 3 * 64];
        for (const Stage &sg_ : l)
          for (int sg = 0; sg < pl.NSTG; ++sg, ++n) {
            if (n >= 60) continue;   // does not fit the per-lane table: counted, not stored
            tab[n] = int32_t((int64_t(sg_.v) * m->c[1] + int64_t(sg) * pl.VC) * m->c[2] * m->c[3]);
            tab[64 + n] = sg_.lo >= 0 ? sg_.lo * pl.NSTG + sg : -1;
            tab[128 + n] = sg_.hi >= 0 ? sg_.hi * pl.NSTG + sg : -1;
          }
        out->counts[(size_t(q) * 2 + x) * 2 + y] = n;
        out->max_wave = std::max(out->max_wave, n);
        out->total_stages += n;
        both += n;
      }
      out->max_stages = std::max(out->max_stages, both);
    }
  }
  out->nq = nq;
  out->ok = out->max_wave <= 60;
}

// Packed layouts.
//  GENERIC: canonical order, nnz elements.
//  MFMA:    [u_o][j_o][v_r][u_i][rb][ch][b][i] with b the position inside a
//           16-wide chunk of the group's (j_i, v_b) contraction list and i the
//           row inside a 4-row block of the group's (u_r, u_b) rows; padding
//           (kk >= KS or row >= R) is zero.  One (u_o, j_o, v_r) slice is the
//           compact W tile of one step of Algorithm 1's outer loop.
//  MFMA_REG: [u_o][j_o][stage][u_i][q][g][i][w]: the stage's contraction list
//           kk = ((v_r % VC) * d_i + j_i) * |G_b.V| + v_b is dealt to 4 lane
//           groups g; element (q, g, i, w) is the weight of row i (< RS, the
//           group's (u_r, u_b) rows padded to a power of two) at position kk = 16q + 4w + g
//           (= step rbgp_reg_step(kk) of the list), so that one 16-byte load per lane
//           fetches a row's weights for four consecutive load slots.
//  MFMA_REG, bf16: same fragment order; the stage's contraction list is cut into blocks
//           of 32 steps and possibly one last block of 16; element (q, g, i, e) of a
//           fragment, e = 0..7, is the weight of row i at kk = 32q + 8g + e in a block of
//           32 and at kk = 32q + 4g + e (e < 4; the rest is padding) in the block of 16:
//           the consecutive contraction steps one lane feeds to the matrix core.
void rbgp_build_pack_perm(const rbgp_mask *m, int kernel, bool bf16, std::vector<int32_t> &perm) {
  if (kernel == RBGP_KERNEL_MFMA_REG && m->regroup && (!bf16 || m->regroup_bf16)) {   // the register layout of the regrouped mask
    rbgp_build_pack_perm(m->regroup, kernel, bf16, perm);         //   (same kept values, same canonical indices)
    return;
  }
  if (kernel == RBGP_KERNEL_MFMA_REG_FILLED) {
    // the register family's layout of the filled mask; a position that holds kept value (row, (j_o, v_r, v_i, v_b))
    // of the filled mask takes this mask's value at (j_o, v_r, j_i, v_b) where v_i = adj_i[u_i][j_i], else a zero
    const rbgp_mask *t = m->filled;
    rbgp_build_pack_perm(t, RBGP_KERNEL_MFMA_REG, bf16, perm);
    if (m->filled_kind == 1) {
      // G_o filled in and merged with G_r: the filled mask's kept value (row, (v_o c_r + v_r, j_i, v_b)) is this mask's
      // value at (j_o, j_r, j_i, j_b) with v_o = adj_o[u_o][j_o] (v_r, v_b likewise), else a zero
      std::vector<int32_t> wh[4];
      for (int i : {0, 1, 3}) {
        wh[i].assign(size_t(m->a[i]) * m->c[i], -1);
        for (int u = 0; u < m->a[i]; ++u)
          for (int j = 0; j < m->d[i]; ++j) wh[i][size_t(u) * m->c[i] + m->adj[i][size_t(u) * m->d[i] + j]] = j;
      }
      const int64_t c3 = m->c[3], d2 = m->d[2], c1 = m->c[1];
      const int64_t rows_o = int64_t(m->a[1]) * m->a[2] * m->a[3], rows_r = int64_t(m->a[2]) * m->a[3];
      for (int32_t &s : perm) {
        if (s < 0) continue;
        const int64_t row = s / t->rowdeg, tt = s % t->rowdeg;
        const int64_t v4 = tt % c3, j3 = (tt / c3) % d2, vr = tt / (c3 * d2);
        const int64_t v1 = vr / c1, v2 = vr % c1;
        const int64_t u1 = row / rows_o, u2 = (row / rows_r) % m->a[1], u4 = row % m->a[3];
        const int j1 = wh[0][size_t(u1 * m->c[0] + v1)], j2 = wh[1][size_t(u2 * c1 + v2)], j4 = wh[3][size_t(u4 * c3 + v4)];
        s = j1 < 0 ? -1 : int32_t(row * m->rowdeg + ((int64_t(j1) * m->d[1] + j2) * d2 + j3) * m->d[3] + j4);
      }
      return;
    }
    std::vector<int32_t> where(size_t(m->a[2]) * m->c[2], -1);   // where[u_i * c_i + v_i]: position of v_i in adj_i[u_i]
    for (int u = 0; u < m->a[2]; ++u)
      for (int j = 0; j < m->d[2]; ++j) where[size_t(u) * m->c[2] + m->adj[2][size_t(u) * m->d[2] + j]] = j;
    const int64_t c2 = m->c[2], c3 = m->c[3], crf = int64_t(m->c[1]) * c2;
    for (int32_t &s : perm) {
      if (s < 0) continue;
      const int64_t row = s / t->rowdeg, tt = s % t->rowdeg;
      const int64_t v4 = tt % c3, vr = (tt / c3) % crf, j1 = tt / (c3 * crf);
      const int64_t v2 = vr / c2, v3 = vr % c2, u3 = (row / m->a[3]) % m->a[2];
      const int j3 = where[size_t(u3 * c2 + v3)];
      s = j3 < 0 ? -1 : int32_t(row * m->rowdeg + ((j1 * m->c[1] + v2) * m->d[2] + j3) * c3 + v4);
    }
    return;
  }
  if (kernel == RBGP_KERNEL_MFMA_TILE) {
    // [u_o][j_o][c][h][row][e]: element e = 0..7 is the weight of row `row` of the tile at tile column
    // 16c + 8h + e (the eight consecutive contraction steps one lane feeds to a 16-step MFMA); tile column
    // (v_r * |G_i.V| + v_i) * |G_b.V| + v_b; zero where an inner graph has no edge and past TK.
    const rbgp_tile_plan p = rbgp_plan_tile(m);
    perm.assign(size_t(p.packed_elems), -1);
    std::vector<int32_t> where[4];   // where[i][u * c_i + v]: position of v in adj_i[u], -1: no edge
    for (int i = 1; i < 4; ++i) {
      where[i].assign(size_t(m->a[i]) * m->c[i], -1);
      for (int u = 0; u < m->a[i]; ++u)
        for (int j = 0; j < m->d[i]; ++j) where[i][size_t(u) * m->c[i] + m->adj[i][size_t(u) * m->d[i] + j]] = j;
    }
    size_t pos = 0;
    for (int u1 = 0; u1 < m->a[0]; ++u1)
      for (int j1 = 0; j1 < m->d[0]; ++j1)
        for (int c = 0; c < p.TKP / 16; ++c)
          for (int h = 0; h < 2; ++h)
            for (int row = 0; row < p.TM; ++row)
              for (int e = 0; e < 8; ++e, ++pos) {
                const int kk = 16 * c + 8 * h + e;
                if (kk >= p.TK) continue;
                const int v4 = kk % m->c[3], v3 = (kk / m->c[3]) % m->c[2], v2 = kk / (m->c[3] * m->c[2]);
                const int u4 = row % m->a[3], u3 = (row / m->a[3]) % m->a[2], u2 = row / (m->a[3] * m->a[2]);
                const int j2 = where[1][size_t(u2) * m->c[1] + v2], j3 = where[2][size_t(u3) * m->c[2] + v3],
                          j4 = where[3][size_t(u4) * m->c[3] + v4];
                if (j2 < 0 || j3 < 0 || j4 < 0) continue;
                const int64_t t = ((int64_t(j1) * m->d[1] + j2) * m->d[2] + j3) * m->d[3] + j4;
                perm[pos] = int32_t((int64_t(u1) * p.TM + row) * m->rowdeg + t);
              }
    return;
  }
  if (kernel == RBGP_KERNEL_MFMA_REG && bf16) {
    const rbgp_reg_plan &p = m->reg;
    const int a1 = p.TR, a2 = p.A2, a3 = m->a[2], a4 = m->a[3], d1 = m->d[0];
    const int nk32 = rbgp_bf16_blocks32(p.KC);
    const int nq = nk32 + (rbgp_bf16_tail16(p.KC) ? 1 : 0);
    perm.assign(size_t(p.packed_elems_bf16), -1);
    size_t pos = 0;
    for (int u1 = 0; u1 < a1; ++u1)
      for (int j1 = 0; j1 < d1; ++j1)
        for (int sg = 0; sg < p.NSTG; ++sg)
          for (int u3 = 0; u3 < a3; ++u3)
            for (int q = 0; q < nq; ++q)
              for (int g = 0; g < 4; ++g)
                for (int r = 0; r < p.RS; ++r)
                  for (int e = 0; e < 8; ++e, ++pos) {
                    if (q >= nk32 && e >= 4) continue;   // upper half of the block of 16: padding
                    const int kk = q < nk32 ? 32 * q + 8 * g + e : 32 * q + 4 * g + e;
                    if (kk >= p.KCR || r >= p.R) continue;
                    const int u2 = r / a4, u4 = r % a4;
                    const int64_t row = ((int64_t(u1) * a2 + u2) * a3 + u3) * a4 + u4;
                    const int64_t t = int64_t(j1) * p.KT + int64_t(sg) * p.KCR + kk;
                    perm[pos] = int32_t(row * m->rowdeg + t);
                  }
    return;
  }
  if (kernel == RBGP_KERNEL_MFMA_REG) {
    const rbgp_reg_plan &p = m->reg;
    const int a1 = p.TR, a2 = p.A2, a3 = m->a[2], a4 = m->a[3], d1 = m->d[0];
    perm.assign(size_t(p.packed_elems), -1);
    size_t pos = 0;
    for (int u1 = 0; u1 < a1; ++u1)
      for (int j1 = 0; j1 < d1; ++j1)
        for (int sg = 0; sg < p.NSTG; ++sg)
          for (int u3 = 0; u3 < a3; ++u3)
            for (int q = 0; q < p.NQ; ++q)
              for (int g = 0; g < 4; ++g)
                for (int r = 0; r < p.RS; ++r)
                  for (int w = 0; w < 4; ++w, ++pos) {
                    const int kk = 16 * q + 4 * w + g;
                    if (kk >= p.KCR || r >= p.R) continue;
                    const int u2 = r / a4, u4 = r % a4;
                    const int64_t row = ((int64_t(u1) * a2 + u2) * a3 + u3) * a4 + u4;
                    const int64_t t = int64_t(j1) * p.KT + int64_t(sg) * p.KCR + rbgp_reg_step(m, kk);
                    perm[pos] = int32_t(row * m->rowdeg + t);
                  }
    return;
  }
  if (kernel != RBGP_KERNEL_MFMA) {
    perm.resize(size_t(m->nnz));
    for (int64_t i = 0; i < m->nnz; ++i) perm[size_t(i)] = int32_t(i);
    return;
  }
  const rbgp_mfma_plan &p = m->plan;
  const int a1 = m->a[0], a2 = m->a[1], a3 = m->a[2], a4 = m->a[3];
  const int d1 = m->d[0], d2 = m->d[1], d3 = m->d[2], d4 = m->d[3];
  perm.assign(size_t(p.packed_elems), -1);
  size_t pos = 0;
  for (int u1 = 0; u1 < a1; ++u1)
    for (int j1 = 0; j1 < d1; ++j1)
      for (int v2 = 0; v2 < d2; ++v2)
        for (int u3 = 0; u3 < a3; ++u3)
          for (int rb = 0; rb < p.RB; ++rb)
            for (int ch = 0; ch < p.NCH; ++ch)
              for (int b = 0; b < 16; ++b)
                for (int i = 0; i < 4; ++i, ++pos) {
                  const int kk = ch * 16 + b, r = rb * 4 + i;
                  if (kk >= p.KS || r >= p.R) continue;
                  const int j3 = kk / d4, v4 = kk % d4;
                  const int u2 = r / a4, u4 = r % a4;
                  const int64_t row = ((int64_t(u1) * a2 + u2) * a3 + u3) * a4 + u4;
                  const int64_t t = ((int64_t(j1) * d2 + v2) * d3 + j3) * d4 + v4;
                  perm[pos] = int32_t(row * m->rowdeg + t);
                }
}

extern "C" {

// Sample one base graph (Appendix "Ramanujan Bipartite Graph Generation"): complete when d == c, else
// 2-lifts of a complete graph, resampled with coin stream (seed, index, attempt) until Ramanujan.
static int sample_base(int a, int c, int d, uint64_t seed, int index, int max_tries, rbgp_base_graph *g) {
  if (a <= 0 || c <= 0 || d <= 0 || d > c || c % d) return RBGP_EINVAL;
  const int lifts = ilog2_exact(c / d);
  if (lifts < 0 || a % (1 << lifts)) return RBGP_EINVAL;
  const int e = int(int64_t(a) * d / c);
  g->a = a; g->c = c; g->d = d; g->e = e;
  g->bound = std::sqrt(double(d - 1)) + std::sqrt(double(e - 1));
  Bits B;
  if (d == c) {
    B.assign(size_t(a) * c, 1);
    g->sigma1 = std::sqrt(double(a) * c);
    g->sigma2 = 0;
    g->status = RBGP_SPEC_COMPLETE;
    g->tries = 0;
  } else {
    bool accepted = false;
    for (int t = 0; t < max_tries && !accepted; ++t) {
      Coins coins(seed, uint64_t(index), uint64_t(t));
      B = sample_biregular(a, c, lifts, coins);
      top_singular(B, a, c, d, e, g->bound, &g->sigma1, &g->sigma2);
      g->tries = t + 1;
      if (std::min(d, e) == 1) {
        g->status = RBGP_SPEC_DEGENERATE;
        accepted = true;
      } else if (g->sigma2 <= g->bound * (1.0 + 1e-9)) {
        g->status = RBGP_SPEC_OK;
        accepted = true;
      }
    }
    if (!accepted) return RBGP_ENOTRAMANUJAN;
  }
  g->adj.resize(size_t(a) * d);
  for (int u = 0; u < a; ++u) {
    int j = 0;
    for (int v = 0; v < c; ++v)
      if (B[size_t(u) * c + v]) g->adj[size_t(u) * d + j++] = v;
  }
  return RBGP_OK;
}

// Factor `role` of the four-factor mask = the product of the base graphs of that role, in order
// (Section 3: the product's biadjacency matrix is the Kronecker product of theirs).  Vertex tuples
// are numbered with the last graph fastest; the neighbours of a tuple are the tuples of neighbours
// in lexicographic order, which ascends because every list ascends.
static void merge_role(rbgp_mask *m, int role) {
  int32_t a = 1, c = 1, d = 1, e = 1;
  std::vector<int32_t> adj(1, 0);   // the trivial graph on (1, 1) vertices
  double s1 = 1, s2 = 0;
  int count = 0, status = RBGP_SPEC_COMPLETE, tries = 0;
  bool all_complete = true, degenerate = false;
  for (const rbgp_base_graph &g : m->base) {
    if (g.role != role) continue;
    std::vector<int32_t> next(size_t(a) * g.a * d * g.d);
    for (int u = 0; u < a; ++u)
      for (int ug = 0; ug < g.a; ++ug)
        for (int j = 0; j < d; ++j)
          for (int jg = 0; jg < g.d; ++jg)
            next[(size_t(u) * g.a + ug) * d * g.d + size_t(j) * g.d + jg] =
                adj[size_t(u) * d + j] * g.c + g.adj[size_t(ug) * g.d + jg];
    adj.swap(next);
    // singular values of a Kronecker product are the products of the factors' singular values
    s2 = std::max(s2 * g.sigma1, s1 * g.sigma2);
    s1 *= g.sigma1;
    a *= g.a; c *= g.c; d *= g.d; e *= g.e;
    all_complete = all_complete && g.status == RBGP_SPEC_COMPLETE;
    degenerate = degenerate || g.status == RBGP_SPEC_DEGENERATE;
    status = g.status;
    tries += g.tries;
    ++count;
  }
  if (count > 1) status = all_complete ? RBGP_SPEC_COMPLETE : degenerate ? RBGP_SPEC_DEGENERATE : RBGP_SPEC_PRODUCT;
  m->a[role] = a; m->c[role] = c; m->d[role] = d; m->e[role] = e;
  m->adj[role].swap(adj);
  m->sigma1[role] = s1; m->sigma2[role] = s2;
  m->bound[role] = std::sqrt(double(d - 1)) + std::sqrt(double(e - 1));
  m->status[role] = status; m->tries[role] = tries;
}

int rbgp_make_mask_k(int32_t count, const int32_t *rows, const int32_t *cols, const int32_t *row_deg,
                     const int32_t *roles, uint64_t seed, int32_t max_tries, rbgp_mask_t **out) {
  if (!rows || !cols || !row_deg || !roles || !out || count < 1 || count > 16) return RBGP_EINVAL;
  if (max_tries <= 0) max_tries = 1000;
  int64_t M = 1, K = 1, rowdeg = 1, coldeg = 1;
  for (int i = 0; i < count; ++i) {
    if (rows[i] <= 0 || cols[i] <= 0 || row_deg[i] <= 0 || row_deg[i] > cols[i]) return RBGP_EINVAL;
    if (roles[i] < 0 || roles[i] > 3 || (i && roles[i] < roles[i - 1])) return RBGP_EINVAL;
    M *= rows[i];
    K *= cols[i];
    rowdeg *= row_deg[i];
    coldeg *= int64_t(rows[i]) * row_deg[i] / cols[i];
    if (M > (1 << 24) || K > (1 << 24)) return RBGP_EINVAL;
  }
  if (M * rowdeg >= (int64_t(1) << 31)) return RBGP_EINVAL;
  rbgp_mask *m = new (std::nothrow) rbgp_mask();
  if (!m) return RBGP_ENOMEM;
  try {
    m->base.resize(size_t(count));
    for (int i = 0; i < count; ++i) {
      m->base[size_t(i)].role = roles[i];
      const int rc = sample_base(rows[i], cols[i], row_deg[i], seed, i, max_tries, &m->base[size_t(i)]);
      if (rc) {
        delete m;
        return rc;
      }
    }
    // The kernels' view wants the factors of roles 1 and 3 complete (Section 5: G_r and G_b).  Where the
    // caller's grouping has a sparse graph there, the graphs of that role up to its last sparse one join
    // the role before (0 or 2), which may be sparse; by associativity the mask, its canonical order and
    // M, K do not change.  rbgp_mask_base keeps reporting the role the caller gave.
    std::vector<int32_t> given(static_cast<size_t>(count), 0);
    for (int i = 0; i < count; ++i) given[size_t(i)] = m->base[size_t(i)].role;
    for (int role : {1, 3}) {
      int last_sparse = -1;
      for (int i = 0; i < count; ++i)
        if (m->base[size_t(i)].role == role && m->base[size_t(i)].status != RBGP_SPEC_COMPLETE) last_sparse = i;
      for (int i = 0; i <= last_sparse; ++i)
        if (m->base[size_t(i)].role == role) m->base[size_t(i)].role = role - 1;
    }
    // A complete G_i is row repetition like G_r (Section 5: every row of the block has the same columns), and the
    // kernels make more of it there: rows that share a column set fill the 16 rows of an MFMA group without
    // pairing tile rows that share only some of their tiles.  So where every graph in the role of G_i is complete,
    // they join G_r in the kernels' view (G_i becomes the single-vertex graph).
    {
      bool any = false, all_complete = true;
      for (int i = 0; i < count; ++i)
        if (m->base[size_t(i)].role == 2) {
          any = true;
          all_complete = all_complete && m->base[size_t(i)].status == RBGP_SPEC_COMPLETE;
        }
      if (any && all_complete)
        for (int i = 0; i < count; ++i)
          if (m->base[size_t(i)].role == 2) m->base[size_t(i)].role = 1;
    }
    for (int role = 0; role < 4; ++role) merge_role(m, role);
    for (int i = 0; i < count; ++i) m->base[size_t(i)].role = given[size_t(i)];
  } catch (const std::bad_alloc &) {
    delete m;
    return RBGP_ENOMEM;
  }
  m->M = M; m->K = K; m->rowdeg = rowdeg; m->coldeg = coldeg; m->nnz = M * rowdeg;
  m->kernel_choice = RBGP_KERNEL_AUTO;
  m->uid = rbgp_next_uid();
  m->dev = nullptr;
  try {   // (the plans allocate their host tables)
    rbgp_plan_mfma(m);
    rbgp_plan_reg(m);
    rbgp_plan_filled(m);
    rbgp_plan_regroup(m);
  } catch (const std::bad_alloc &) {
    rbgp_mask_free(m);
    return RBGP_ENOMEM;
  } catch (...) {
    rbgp_mask_free(m);
    return RBGP_EINTERNAL;
  }
  *out = m;
  return RBGP_OK;
}

int rbgp_make_mask(const int32_t rows[4], const int32_t cols[4], const int32_t row_deg[4],
                   uint64_t seed, int32_t max_tries, rbgp_mask_t **out) {
  static const int32_t roles[4] = {0, 1, 2, 3};
  return rbgp_make_mask_k(4, rows, cols, row_deg, roles, seed, max_tries, out);
}

int rbgp_mask_num_base(const rbgp_mask_t *m) { return m ? int(m->base.size()) : RBGP_EINVAL; }

int rbgp_mask_base(const rbgp_mask_t *m, int i, int32_t *rows, int32_t *cols, int32_t *deg, int32_t *role,
                   const int32_t **adj, double *sigma1, double *sigma2, double *bound, int *status, int *tries) {
  if (!m || i < 0 || i >= int(m->base.size())) return RBGP_EINVAL;
  const rbgp_base_graph &g = m->base[size_t(i)];
  if (rows) *rows = g.a;
  if (cols) *cols = g.c;
  if (deg) *deg = g.d;
  if (role) *role = g.role;
  if (adj) *adj = g.adj.data();
  if (sigma1) *sigma1 = g.sigma1;
  if (sigma2) *sigma2 = g.sigma2;
  if (bound) *bound = g.bound;
  if (status) *status = g.status;
  if (tries) *tries = g.tries;
  return RBGP_OK;
}

// The s-th kept value of W_s^T (row k of the transpose, positions in the order of the
// co-adjacency lists, i.e. ascending original row) is the kept value (row, t) of W_s, t being the
// position of k's factor vertices in the adjacency lists of the row's factor vertices.
static void transposed_order(const rbgp_mask *m, const std::vector<int32_t> coadj[4], int32_t *out) {
  std::vector<int32_t> pos[4];   // pos[i][u * c + v] = position of v in adj[i][u], -1: not adjacent
  for (int i = 0; i < 4; ++i) {
    pos[i].assign(size_t(m->a[i]) * m->c[i], -1);
    for (int u = 0; u < m->a[i]; ++u)
      for (int j = 0; j < m->d[i]; ++j) pos[i][size_t(u) * m->c[i] + m->adj[i][size_t(u) * m->d[i] + j]] = j;
  }
  const int32_t *a = m->a, *c = m->c, *d = m->d, *e = m->e;
  int64_t s = 0;
  for (int v0 = 0; v0 < c[0]; ++v0)
    for (int v1 = 0; v1 < c[1]; ++v1)
      for (int v2 = 0; v2 < c[2]; ++v2)
        for (int v3 = 0; v3 < c[3]; ++v3)
          for (int j0 = 0; j0 < e[0]; ++j0)
            for (int j1 = 0; j1 < e[1]; ++j1)
              for (int j2 = 0; j2 < e[2]; ++j2)
                for (int j3 = 0; j3 < e[3]; ++j3) {
                  const int u0 = coadj[0][size_t(v0) * e[0] + j0], u1 = coadj[1][size_t(v1) * e[1] + j1],
                            u2 = coadj[2][size_t(v2) * e[2] + j2], u3 = coadj[3][size_t(v3) * e[3] + j3];
                  const int64_t row = ((int64_t(u0) * a[1] + u1) * a[2] + u2) * a[3] + u3;
                  const int64_t t = ((int64_t(pos[0][size_t(u0) * c[0] + v0]) * d[1] + pos[1][size_t(u1) * c[1] + v1]) * d[2] +
                                     pos[2][size_t(u2) * c[2] + v2]) * d[3] + pos[3][size_t(u3) * c[3] + v3];
                  out[s++] = int32_t(row * m->rowdeg + t);
                }
}

static void co_adjacency(const rbgp_mask *m, std::vector<int32_t> coadj[4]) {
  for (int i = 0; i < 4; ++i) {
    coadj[i].assign(size_t(m->c[i]) * m->e[i], 0);
    std::vector<int> fill(size_t(m->c[i]), 0);
    for (int u = 0; u < m->a[i]; ++u)       // ascending u: every list ascends
      for (int j = 0; j < m->d[i]; ++j) {
        const int v = m->adj[i][size_t(u) * m->d[i] + j];
        coadj[i][size_t(v) * m->e[i] + fill[size_t(v)]++] = u;
      }
  }
}

static int transpose_order_impl(const rbgp_mask_t *m, int32_t *out) {
  if (!m || !out) return RBGP_EINVAL;
  try {
    std::vector<int32_t> coadj[4];
    co_adjacency(m, coadj);
    transposed_order(m, coadj, out);
  } catch (const std::bad_alloc &) {
    return RBGP_ENOMEM;
  }
  return RBGP_OK;
}

int rbgp_transpose_order(const rbgp_mask_t *m, int32_t *out) {
  RBGP_GUARDED(transpose_order_impl(m, out));
}

int rbgp_mask_transpose(const rbgp_mask_t *m, rbgp_mask_t **out) {
  if (!m || !out) return RBGP_EINVAL;
  if (m->K * m->coldeg >= (int64_t(1) << 31)) return RBGP_EINVAL;
  rbgp_mask *t = new (std::nothrow) rbgp_mask();
  if (!t) return RBGP_ENOMEM;
  try {
    std::vector<int32_t> coadj[4];
    co_adjacency(m, coadj);
    for (int i = 0; i < 4; ++i) {
      t->a[i] = m->c[i]; t->c[i] = m->a[i]; t->d[i] = m->e[i]; t->e[i] = m->d[i];
      t->sigma1[i] = m->sigma1[i]; t->sigma2[i] = m->sigma2[i]; t->bound[i] = m->bound[i];   // singular values of B^T are B's
      t->status[i] = m->status[i]; t->tries[i] = m->tries[i];
    }
    for (const rbgp_base_graph &g : m->base) {   // the transposed base graphs, for introspection
      rbgp_base_graph gt;
      gt.a = g.c; gt.c = g.a; gt.d = g.e; gt.e = g.d; gt.role = g.role;
      gt.sigma1 = g.sigma1; gt.sigma2 = g.sigma2; gt.bound = g.bound; gt.status = g.status; gt.tries = g.tries;
      gt.adj.assign(size_t(g.c) * g.e, 0);
      std::vector<int> fill(size_t(g.c), 0);
      for (int u = 0; u < g.a; ++u)
        for (int j = 0; j < g.d; ++j) {
          const int v = g.adj[size_t(u) * g.d + j];
          gt.adj[size_t(v) * g.e + fill[size_t(v)]++] = u;
        }
      t->base.push_back(std::move(gt));
    }
    t->from_original.resize(size_t(m->nnz));
    transposed_order(m, coadj, t->from_original.data());
    for (int i = 0; i < 4; ++i) t->adj[i] = std::move(coadj[i]);
    t->M = m->K; t->K = m->M; t->rowdeg = m->coldeg; t->coldeg = m->rowdeg; t->nnz = m->nnz;
    t->kernel_choice = RBGP_KERNEL_AUTO;
    t->uid = rbgp_next_uid();
    t->dev = nullptr;
    rbgp_plan_mfma(t);
    rbgp_plan_reg(t);
    rbgp_plan_filled(t);
    rbgp_plan_regroup(t);
  } catch (const std::bad_alloc &) {
    delete t;
    return RBGP_ENOMEM;
  }
  *out = t;
  return RBGP_OK;
}

// The mask of the transposed 3x3 convolution.  O = W_s x im2col(X) means
//   O[m][y][x] = sum_{c, dy, dx} W[m][9c + 3(dy+1) + (dx+1)] X[c][y+dy][x+dx],
// so the gradient with respect to X is again a 3x3 convolution, of dO:
//   dX[c][y][x] = sum_{m, dy', dx'} W'[c][9m + 3(dy'+1) + (dx'+1)] dO[m][y+dy'][x+dx'],
//   W'[c][9m + tap'] = W[m][9c + (8 - tap')]            (dy' = -dy, dx' = -dx).
// Its mask over rows c = (v_o, v_r, v_i) and columns (u_o, u_r, u_i, u_b, tap') is
//   G_o^T (x) G_r^T (x) (G_i^T (x) J(1, |G_b.U|)) (x) J(1, 9)
// with J(a, c) the complete graph: a four-factor mask of the same family (G_b complete makes every
// (u_b, tap') adjacent to every row), with the nine taps innermost as the fused kernel wants them.
int rbgp_mask_conv3x3_transpose(const rbgp_mask_t *m, rbgp_mask_t **out) {
  if (!m || !out) return RBGP_EINVAL;
  if (m->c[3] != 9 || m->d[3] != 9) return RBGP_EUNSUPPORTED;
  if ((m->K / 9) * (m->coldeg * 9) >= (int64_t(1) << 31) || m->M * 9 > (1 << 24)) return RBGP_EINVAL;
  rbgp_mask *t = new (std::nothrow) rbgp_mask();
  if (!t) return RBGP_ENOMEM;
  try {
    std::vector<int32_t> coadj[4];
    co_adjacency(m, coadj);
    const int ab = m->a[3];
    for (int i = 0; i < 3; ++i) {
      rbgp_base_graph g;
      g.a = m->c[i]; g.c = m->a[i]; g.d = m->e[i]; g.e = m->d[i]; g.role = i;
      g.adj = coadj[i];
      g.sigma1 = m->sigma1[i]; g.sigma2 = m->sigma2[i]; g.bound = m->bound[i];
      g.status = m->status[i]; g.tries = m->tries[i];
      t->base.push_back(std::move(g));
    }
    for (int i = 0; i < 2; ++i) {   // J(1, |G_b.U|) joins G_i^T; J(1, 9) are the taps
      rbgp_base_graph g;
      g.a = 1; g.c = i ? 9 : ab; g.d = g.c; g.e = 1; g.role = i ? 3 : 2;
      g.adj.resize(size_t(g.c));
      for (int v = 0; v < g.c; ++v) g.adj[size_t(v)] = v;
      g.sigma1 = std::sqrt(double(g.c)); g.sigma2 = 0; g.bound = std::sqrt(double(g.c - 1));
      g.status = RBGP_SPEC_COMPLETE; g.tries = 0;
      t->base.push_back(std::move(g));
    }
    for (int role = 0; role < 4; ++role) merge_role(t, role);
    t->M = m->K / 9; t->K = m->M * 9;
    t->rowdeg = int64_t(t->d[0]) * t->d[1] * t->d[2] * t->d[3];
    t->coldeg = int64_t(t->e[0]) * t->e[1] * t->e[2] * t->e[3];
    t->nnz = m->nnz;
    // where each kept value of W' comes from
    std::vector<int32_t> pos[3];
    for (int i = 0; i < 3; ++i) {
      pos[i].assign(size_t(m->a[i]) * m->c[i], -1);
      for (int u = 0; u < m->a[i]; ++u)
        for (int j = 0; j < m->d[i]; ++j) pos[i][size_t(u) * m->c[i] + m->adj[i][size_t(u) * m->d[i] + j]] = j;
    }
    t->from_original.resize(size_t(m->nnz));
    const int32_t *a = m->a, *c = m->c, *d = m->d, *e = m->e;
    int64_t s = 0;
    for (int v0 = 0; v0 < c[0]; ++v0)
      for (int v1 = 0; v1 < c[1]; ++v1)
        for (int v2 = 0; v2 < c[2]; ++v2)
          for (int j0 = 0; j0 < e[0]; ++j0)
            for (int j1 = 0; j1 < e[1]; ++j1)
              for (int j2 = 0; j2 < e[2]; ++j2)
                for (int ub = 0; ub < ab; ++ub)
                  for (int tap = 0; tap < 9; ++tap) {
                    const int u0 = coadj[0][size_t(v0) * e[0] + j0], u1 = coadj[1][size_t(v1) * e[1] + j1],
                              u2 = coadj[2][size_t(v2) * e[2] + j2];
                    const int64_t row = ((int64_t(u0) * a[1] + u1) * a[2] + u2) * ab + ub;
                    const int64_t at = ((int64_t(pos[0][size_t(u0) * c[0] + v0]) * d[1] + pos[1][size_t(u1) * c[1] + v1]) * d[2] +
                                        pos[2][size_t(u2) * c[2] + v2]) * 9 + (8 - tap);
                    t->from_original[size_t(s++)] = int32_t(row * m->rowdeg + at);
                  }
    t->kernel_choice = RBGP_KERNEL_AUTO;
    t->uid = rbgp_next_uid();
    t->dev = nullptr;
    rbgp_plan_mfma(t);
    rbgp_plan_reg(t);
    rbgp_plan_filled(t);
    rbgp_plan_regroup(t);
  } catch (const std::bad_alloc &) {
    delete t;
    return RBGP_ENOMEM;
  }
  *out = t;
  return RBGP_OK;
}

static int mask_original_order_impl(const rbgp_mask_t *m, int32_t *out) {
  if (!m || !out || m->from_original.empty()) return RBGP_EINVAL;
  std::copy(m->from_original.begin(), m->from_original.end(), out);
  return RBGP_OK;
}

int rbgp_mask_original_order(const rbgp_mask_t *m, int32_t *out) {
  RBGP_GUARDED(mask_original_order_impl(m, out));
}

void rbgp_mask_free(rbgp_mask_t *mask) {
  if (!mask) return;
  if (mask->dev) rbgp_device_release(mask->dev);
  if (mask->filled) rbgp_mask_free(mask->filled);
  if (mask->regroup) rbgp_mask_free(mask->regroup);
  delete mask;
}

int rbgp_mask_shape(const rbgp_mask_t *m, int64_t *M, int64_t *K, int64_t *rowdeg, int64_t *coldeg,
                    int64_t *nnz) {
  if (!m) return RBGP_EINVAL;
  if (M) *M = m->M;
  if (K) *K = m->K;
  if (rowdeg) *rowdeg = m->rowdeg;
  if (coldeg) *coldeg = m->coldeg;
  if (nnz) *nnz = m->nnz;
  return RBGP_OK;
}

int rbgp_mask_factor(const rbgp_mask_t *m, int i, int32_t *rows, int32_t *cols, int32_t *deg,
                     const int32_t **adj) {
  if (!m || i < 0 || i > 3) return RBGP_EINVAL;
  if (rows) *rows = m->a[i];
  if (cols) *cols = m->c[i];
  if (deg) *deg = m->d[i];
  if (adj) *adj = m->adj[i].data();
  return RBGP_OK;
}

int rbgp_mask_spectrum(const rbgp_mask_t *m, int i, double *sigma1, double *sigma2, double *bound,
                       int *status, int *tries) {
  if (!m || i < 0 || i > 3) return RBGP_EINVAL;
  if (sigma1) *sigma1 = m->sigma1[i];
  if (sigma2) *sigma2 = m->sigma2[i];
  if (bound) *bound = m->bound[i];
  if (status) *status = m->status[i];
  if (tries) *tries = m->tries[i];
  return RBGP_OK;
}

static int mask_columns_impl(const rbgp_mask_t *m, int32_t *out) {
  if (!m || !out) return RBGP_EINVAL;
  const int32_t *A0 = m->adj[0].data(), *A1 = m->adj[1].data(), *A2 = m->adj[2].data(),
                *A3 = m->adj[3].data();
  int64_t pos = 0;
  for (int u0 = 0; u0 < m->a[0]; ++u0)
    for (int u1 = 0; u1 < m->a[1]; ++u1)
      for (int u2 = 0; u2 < m->a[2]; ++u2)
        for (int u3 = 0; u3 < m->a[3]; ++u3)
          for (int j0 = 0; j0 < m->d[0]; ++j0)
            for (int j1 = 0; j1 < m->d[1]; ++j1)
              for (int j2 = 0; j2 < m->d[2]; ++j2)
                for (int j3 = 0; j3 < m->d[3]; ++j3) {
                  int64_t k = A0[u0 * m->d[0] + j0];
                  k = k * m->c[1] + A1[u1 * m->d[1] + j1];
                  k = k * m->c[2] + A2[u2 * m->d[2] + j2];
                  k = k * m->c[3] + A3[u3 * m->d[3] + j3];
                  out[pos++] = int32_t(k);
                }
  return RBGP_OK;
}

int rbgp_mask_columns(const rbgp_mask_t *m, int32_t *out) {
  RBGP_GUARDED(mask_columns_impl(m, out));
}

static int mask_dense_impl(const rbgp_mask_t *m, uint8_t *out) {
  if (!m || !out) return RBGP_EINVAL;
  std::memset(out, 0, size_t(m->M) * size_t(m->K));
  std::vector<int32_t> cols(size_t(m->nnz));
  rbgp_mask_columns(m, cols.data());
  for (int64_t row = 0; row < m->M; ++row)
    for (int64_t t = 0; t < m->rowdeg; ++t)
      out[size_t(row) * size_t(m->K) + size_t(cols[size_t(row * m->rowdeg + t)])] = 1;
  return RBGP_OK;
}

int rbgp_mask_dense(const rbgp_mask_t *m, uint8_t *out) {
  RBGP_GUARDED(mask_dense_impl(m, out));
}

static int mask_reg_plan_impl(const rbgp_mask_t *m, int32_t info[16]) {
  if (!m || !info) return RBGP_EINVAL;
  for (int i = 0; i < 16; ++i) info[i] = 0;
  if (m->filled) info[13] = m->filled->reg_clusters.max_stages;
  if (m->regroup) {   // fp32 runs on the regrouped mask
    info[14] = m->regroup->reg.R;
    info[15] = m->regroup->reg.TR;
  }
  const rbgp_reg_plan &p = m->reg;
  if (!p.ok) return RBGP_OK;
  info[0] = p.MG; info[1] = p.NSTG; info[2] = p.KC; info[3] = p.TR;
  const rbgp_reg_clusters &cl = m->reg_clusters;
  info[4] = cl.ncl; info[5] = cl.max_stages;
  for (int32_t c : cl.counts) info[6] += c;
  const rbgp_reg_dual &d = m->reg_dual;
  if (d.ok) {
    info[7] = d.nq; info[8] = d.max_stages; info[9] = int32_t(d.total_stages); info[10] = d.max_wave;
    // distinct stage bases wanted by the r-th stages of all waves, r = 0 and r <= 1
    std::vector<int32_t> seen;
    for (int r = 0; r < 2; ++r) {
      for (int wv = 0; wv < d.nq * 4; ++wv)
        if (d.counts[size_t(wv)] > r) {
          const int32_t base = d.stages[size_t(wv) * 3 * 64 + r];
          if (std::find(seen.begin(), seen.end(), base) == seen.end()) seen.push_back(base);
        }
      info[11 + r] = int32_t(seen.size());
    }
  }
  return RBGP_OK;
}

int rbgp_mask_reg_plan(const rbgp_mask_t *m, int32_t info[16]) {
  RBGP_GUARDED(mask_reg_plan_impl(m, info));
}

// Every (tile row, tile, stage of the tile) must be multiplied exactly once, by a stage whose base
// row is that tile's, with a fragment position inside the tile row's fragments; stage lists must fit
// their per-lane tables and end in sentinels.
int rbgp_mask_check_tables(const rbgp_mask_t *m) {
  if (!m) return RBGP_EINVAL;
  if (m->filled) {   // the filled mask has tables of its own, and its packed layout must hold every kept value once
    const int rc = rbgp_mask_check_tables(m->filled);
    if (rc) return rc;
    try {
      for (bool bf16 : {false, true}) {
        std::vector<int32_t> perm;
        rbgp_build_pack_perm(m, RBGP_KERNEL_MFMA_REG_FILLED, bf16, perm);
        std::vector<char> seen(size_t(m->nnz), 0);
        for (int32_t s : perm) {
          if (s < -1 || s >= m->nnz) return RBGP_EINTERNAL;
          if (s >= 0 && seen[size_t(s)]++) return RBGP_EINTERNAL;
        }
        for (char c : seen)
          if (!c) return RBGP_EINTERNAL;
      }
    } catch (const std::bad_alloc &) {
      return RBGP_ENOMEM;
    }
  }
  if (m->regroup) {   // the regrouped mask: the same entries in the same order, its own tables, and a packed layout that
                      //   holds every kept value of this mask once
    if (m->regroup->M != m->M || m->regroup->K != m->K || m->regroup->nnz != m->nnz) return RBGP_EINTERNAL;
    const int rc = rbgp_mask_check_tables(m->regroup);
    if (rc) return rc;
    try {
      std::vector<int32_t> mine(size_t(m->nnz)), theirs(size_t(m->nnz));
      if (mask_columns_impl(m, mine.data()) || mask_columns_impl(m->regroup, theirs.data()) || mine != theirs)
        return RBGP_EINTERNAL;
      for (bool bf16 : {false, true}) {
        std::vector<int32_t> perm;
        rbgp_build_pack_perm(m, RBGP_KERNEL_MFMA_REG, bf16, perm);
        std::vector<char> seen(size_t(m->nnz), 0);
        for (int32_t s : perm) {
          if (s < -1 || s >= m->nnz) return RBGP_EINTERNAL;
          if (s >= 0 && seen[size_t(s)]++) return RBGP_EINTERNAL;
        }
        for (char c : seen)
          if (!c) return RBGP_EINTERNAL;
      }
    } catch (const std::bad_alloc &) {
      return RBGP_ENOMEM;
    }
  }
  const rbgp_reg_plan &p = m->reg;
  if (!p.ok) return RBGP_OK;
  try {
    const int d1 = m->d[0], fpm = d1 * p.NSTG;
    const int64_t stage_rows = int64_t(p.VC) * m->c[2] * m->c[3];
    // expected base row of fragment f of tile row u
    auto base_of = [&](int u, int f) {
      const int v = m->adj[0][size_t(u / p.fold) * d1 + f / p.NSTG];
      return (int64_t(v) * m->c[1] + int64_t(f % p.NSTG) * p.VC) * m->c[2] * m->c[3];
    };
    auto check_use = [&](std::vector<int> &used, int u, int f, int64_t base) {
      if (u < 0 || u >= p.TR || f < 0 || f >= fpm) return false;
      if (base != base_of(u, f) || base < 0 || base + stage_rows > m->K) return false;
      return ++used[size_t(u) * fpm + f] == 1;
    };
    {
      const rbgp_reg_clusters &cl = m->reg_clusters;
      std::vector<int> used(size_t(p.TR) * fpm, 0);
      if (cl.max_stages <= kRegMaxStages) {
        const int TS = cl.tstride;
        if (TS != (cl.max_stages > kRegWaveStages ? 256 : 64)) return RBGP_EINTERNAL;
        if (cl.stages.size() != size_t(cl.ncl) * (1 + cl.U) * TS) return RBGP_EINTERNAL;
        for (int c = 0; c < cl.ncl; ++c) {
          const int n = cl.counts[size_t(c)];
          if (n < 0 || n > cl.max_stages) return RBGP_EINTERNAL;
          for (int st = 0; st < TS; ++st) {
            const int32_t base = cl.stages[(size_t(c) * (1 + cl.U)) * TS + st];
            if ((st < n) != (base >= 0)) return RBGP_EINTERNAL;
            for (int k = 0; k < cl.U; ++k) {
              const int32_t f = cl.stages[(size_t(c) * (1 + cl.U) + 1 + k) * TS + st];
              if (st >= n && f != -1) return RBGP_EINTERNAL;
              if (f >= 0 && !check_use(used, cl.members[size_t(c) * cl.U + k], f, base)) return RBGP_EINTERNAL;
            }
          }
        }
        for (int c : used)
          if (c != 1) return RBGP_EINTERNAL;
      }
    }
    // the packed buffer holds exactly the fragments the stage lists can name, plus the zero fragment; the
    // rows of I a stage's contraction steps select lie inside the rows the stage spans
    if (p.packed_elems != (int64_t(p.TR) * fpm * m->a[2] + 1) * p.NQ * 4 * p.RS * 4) return RBGP_EINTERNAL;
    if (p.KCR > p.KC || p.KC > p.NO * 4 || p.NO > p.NQ * 4 || stage_rows != p.SRC) return RBGP_EINTERNAL;
    for (int u3 = 0; u3 < m->a[2]; ++u3)
      for (int kk = 0; kk < p.KCR; ++kk) {
        const int st = rbgp_reg_step(m, kk);
        if (st < 0 || st >= p.KCR) return RBGP_EINTERNAL;
        const int v4 = st % m->c[3], j3 = (st / m->c[3]) % m->d[2], vv = st / (m->c[3] * m->d[2]);
        const int64_t row = (int64_t(vv) * m->c[2] + m->adj[2][size_t(u3) * m->d[2] + j3]) * m->c[3] + v4;
        if (vv >= p.VC || row < 0 || row >= p.SRC) return RBGP_EINTERNAL;
      }
    const rbgp_reg_dual &d = m->reg_dual;
    if (d.ok) {
      std::vector<int> used(size_t(p.TR) * fpm, 0);
      for (int wv = 0; wv < d.nq * 4; ++wv) {
        const int q = wv / 4, x = (wv / 2) % 2, y = wv % 2, n = d.counts[size_t(wv)];
        if (n < 0 || n > 60) return RBGP_EINTERNAL;
        const int32_t *tab = &d.stages[size_t(wv) * 3 * 64];
        for (int st = 0; st < 64; ++st) {
          if ((st < n) != (tab[st] >= 0)) return RBGP_EINTERNAL;
          if (st >= n && (tab[64 + st] != -1 || tab[128 + st] != -1)) return RBGP_EINTERNAL;
          if (tab[64 + st] >= 0 && !check_use(used, d.members[size_t(q) * 4 + x], tab[64 + st], tab[st])) return RBGP_EINTERNAL;
          if (tab[128 + st] >= 0 && !check_use(used, d.members[size_t(q) * 4 + 2 + y], tab[128 + st], tab[st])) return RBGP_EINTERNAL;
        }
      }
      for (int c : used)
        if (c != 1) return RBGP_EINTERNAL;
    }
  } catch (const std::bad_alloc &) {
    return RBGP_ENOMEM;
  }
  return RBGP_OK;
}

const char *rbgp_strerror(int code) {
  switch (code) {
    case RBGP_OK: return "ok";
    case RBGP_EINVAL: return "invalid argument";
    case RBGP_ENOMEM: return "out of memory";
    case RBGP_ENOTRAMANUJAN: return "no Ramanujan sample within max_tries";
    case RBGP_ESHAPE: return "shape, leading dimension or alignment does not match the mask";
    case RBGP_EHIP: return "HIP call failed";
    case RBGP_EUNSUPPORTED: return "kernel does not cover this mask or dtype";
    case RBGP_EINTERNAL: return "an index table of the library is inconsistent";
    case RBGP_ETOOLARGE: return "the problem needs more scratch memory than the allocation-free entry point has";
    default: return "unknown error";
  }
}

const char *rbgp_last_hip_error(void) { return g_hip_error; }

}  // extern "C"
