"""Plain CPU oracle for the RBGP4 product O = W_s x I.  TEST INFRASTRUCTURE ONLY.

Written from the paper alone; shares no code with the HIP library and is
never imported by it.  Everything is numpy float64 / plain Python loops and is
meant to be checked against the paper by eye:

* two_lift, sample_biregular, sample_factor -- Appendix "Ramanujan Bipartite
  Graph Generation" (2-lift operation, sparse biregular generation, RBG
  rejection sampling) with the Ramanujan bound of Section 3.
* kron_mask -- Section 3, bipartite graph product: the biadjacency matrix of a
  product is the tensor (Kronecker) product of the factors' matrices; Section 5
  fixes four factors G_o, G_r, G_i, G_b.
* canonical_columns / scatter_values -- Appendix "Pseudo code for RBGP4MM":
  the kept values of a row are stored as data[rows][(1-sp)*cols]; Algorithm 1
  indexes them by (outk, rk, ink, block column), which is ascending column
  order because every adjacency list ascends.
* spmm_definition -- Section 5 "GPU Implementation": O = W_s x I, written out
  as the masked sum  O[m][n] = sum_k mask[m][k] * W[m][k] * I[k][n]  in float64.
* transpose_order, spmm_transposed_definition, sddmm_definition -- the two
  gradients of that product for a fixed mask (Section 6), as masked sums.

Readings taken where the paper is silent (random source, vertex numbering of a
lift, tie handling of the bound, degenerate factors) are the ones listed in
this repository's design notes; the random source is a counter-based
SplitMix64 stream that the library implements separately from the same
written description.

Pins (tests/ -m "not gpu"): published SplitMix64 outputs; 2-lift invariants;
closed-form singular values (complete graph, 8-cycle, two 4-cycles, star
forest); numpy.kron; degree/density products; the paper's worked examples
(512 edges stored as 22; two factorings giving (64,16) at 75 %); spectrum of a
product; brute-force matmul with explicit zeros; scipy.signal.correlate2d for
the lowered 3x3 convolution; numpy.matmul for all-complete
factors; torch's bf16 conversion for the rounding routine; torch autograd on
the dense masked weight, the adjoint identity and (A (x) B)^T = A^T (x) B^T for
the backward products.
"""
from __future__ import annotations

import math

import numpy as np

_U64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15

STATUS_OK = 0          # sparse factor, passed the Ramanujan test
STATUS_COMPLETE = 1    # complete bipartite factor, nothing sampled
STATUS_DEGENERATE = 2  # min(d_l, d_r) == 1: a star forest, bound unsatisfiable


# --------------------------------------------------------------------------
# random source (the paper only says "chosen at random")
# --------------------------------------------------------------------------
def mix64(z: int) -> int:
    """SplitMix64 output function on a 64-bit integer."""
    z &= _U64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _U64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _U64
    return z ^ (z >> 31)


class CoinStream:
    """Fair coins for (seed, factor index, attempt): coin n = top bit of
    mix64(key + (n+1)*golden), key = mix64(mix64(mix64(seed)+factor)+attempt)."""

    def __init__(self, seed: int, factor: int, attempt: int):
        self.key = mix64(mix64(mix64(seed) + factor) + attempt)
        self.n = 0

    def draw(self) -> int:
        self.n += 1
        return mix64(self.key + self.n * _GOLDEN)

    def coin(self) -> int:
        return self.draw() >> 63


# --------------------------------------------------------------------------
# Appendix: Ramanujan bipartite graph generation
# --------------------------------------------------------------------------
def two_lift(B: np.ndarray, coins: CoinStream) -> np.ndarray:
    """2-lift of the bipartite graph with biadjacency matrix B.

    The lifted graph has the vertices of G and of its clone G^c (clone of u is
    u+|U|, clone of v is v+|V|).  For each edge (u,v), visited with u ascending
    then v ascending, a coin picks the identity pair {(u,v),(u^c,v^c)} (0) or
    the crossover pair {(u,v^c),(u^c,v)} (1)."""
    a, c = B.shape
    out = np.zeros((2 * a, 2 * c), dtype=np.uint8)
    for u in range(a):
        for v in range(c):
            if B[u, v]:
                if coins.coin() == 0:
                    out[u, v] = 1
                    out[u + a, v + c] = 1
                else:
                    out[u, v + c] = 1
                    out[u + a, v] = 1
    return out


def num_lifts(c: int, d: int) -> int:
    """log2(1/(1-sp)) with 1-sp = d/c; raises unless it is a whole number."""
    if d <= 0 or c % d:
        raise ValueError("density d/c is not 1/2^L")
    q = c // d
    if q & (q - 1):
        raise ValueError("density d/c is not 1/2^L")
    return q.bit_length() - 1


def sample_biregular(a: int, c: int, d: int, coins: CoinStream) -> np.ndarray:
    """a x c biregular graph with row degree d: L = log2(c/d) 2-lifts applied
    to the complete bipartite graph on (a/2^L, c/2^L) vertices."""
    L = num_lifts(c, d)
    if a % (1 << L):
        raise ValueError("rows not divisible by 2^L")
    B = np.ones((a >> L, c >> L), dtype=np.uint8)
    for _ in range(L):
        B = two_lift(B, coins)
    return B


def singular_values(B: np.ndarray) -> np.ndarray:
    """Singular values of the biadjacency matrix, descending.  The adjacency
    matrix [[0,B],[B^T,0]] has eigenvalues +-sigma_i, so lambda_2 = sigma_2."""
    return np.linalg.svd(B.astype(np.float64), compute_uv=False)


def ramanujan_bound(d_l: int, d_r: int) -> float:
    """Section 3: lambda_2 <= sqrt(d_l - 1) + sqrt(d_r - 1)."""
    return math.sqrt(d_l - 1) + math.sqrt(d_r - 1)


def second_singular(B: np.ndarray) -> float:
    s = singular_values(B)
    return float(s[1]) if s.size > 1 else 0.0


def sample_factor(a: int, c: int, d: int, seed: int, factor: int, max_tries: int = 1000):
    """One base graph of the product.  d == c is a complete graph (no
    sampling).  Otherwise biregular graphs are sampled, attempt t using coin
    stream (seed, factor, t), until one meets the Ramanujan bound (tested on
    the final graph, accepted iff sigma_2 <= bound*(1+1e-9)).  A factor whose
    smaller degree is 1 can never meet it (a star forest has sigma_2 = sigma_1
    > bound): its first sample is kept and flagged DEGENERATE.

    Returns (B, info) with info = dict(sigma1, sigma2, bound, status, tries)."""
    if d == c:
        B = np.ones((a, c), dtype=np.uint8)
        return B, dict(sigma1=math.sqrt(a * c), sigma2=0.0,
                       bound=ramanujan_bound(c, a), status=STATUS_COMPLETE, tries=0)
    L = num_lifts(c, d)
    if a % (1 << L):
        raise ValueError("rows not divisible by 2^L")
    e = a * d // c
    bound = ramanujan_bound(d, e)
    for t in range(max_tries):
        B = sample_biregular(a, c, d, CoinStream(seed, factor, t))
        s = singular_values(B)
        s2 = float(s[1]) if s.size > 1 else 0.0
        info = dict(sigma1=float(s[0]), sigma2=s2, bound=bound, tries=t + 1)
        if min(d, e) == 1:
            info["status"] = STATUS_DEGENERATE
            return B, info
        if s2 <= bound * (1.0 + 1e-9):
            info["status"] = STATUS_OK
            return B, info
    raise RuntimeError("no Ramanujan sample within max_tries")


def sample_factors(rows, cols, row_deg, seed: int, max_tries: int = 1000):
    """The four base graphs (G_o, G_r, G_i, G_b) of an RBGP4 mask."""
    Bs, infos = [], []
    for i in range(len(rows)):
        B, info = sample_factor(rows[i], cols[i], row_deg[i], seed, i, max_tries)
        Bs.append(B)
        infos.append(info)
    return Bs, infos


def adjacency_lists(B: np.ndarray) -> np.ndarray:
    """adj[u] = ascending neighbours of u; shape (|U|, d_l)."""
    a = B.shape[0]
    deg = int(B[0].sum())
    adj = np.zeros((a, deg), dtype=np.int32)
    for u in range(a):
        nb = np.flatnonzero(B[u])
        assert nb.size == deg, "not row-regular"
        adj[u] = nb
    return adj


# --------------------------------------------------------------------------
# Sections 3-5: the mask
# --------------------------------------------------------------------------
def kron_mask(Bs) -> np.ndarray:
    """Dense biadjacency matrix of G_1 (x)_b ... (x)_b G_K by the definition
    of the product: ((u_1..u_K),(v_1..v_K)) is an edge iff every (u_i,v_i) is.
    Vertex tuples are numbered with the last factor fastest."""
    M = int(np.prod([B.shape[0] for B in Bs]))
    K = int(np.prod([B.shape[1] for B in Bs]))
    mask = np.ones((M, K), dtype=np.uint8)
    m = np.arange(M)
    k = np.arange(K)
    for B in reversed(Bs):
        a, c = B.shape
        u = m % a
        v = k % c
        m = m // a
        k = k // c
        mask &= B[u[:, None], v[None, :]]
    return mask


def canonical_columns(mask: np.ndarray) -> np.ndarray:
    """cols[m][t] = column of the t-th kept value of row m (ascending)."""
    M = mask.shape[0]
    rowdeg = int(mask[0].sum())
    cols = np.zeros((M, rowdeg), dtype=np.int32)
    for m in range(M):
        nz = np.flatnonzero(mask[m])
        assert nz.size == rowdeg, "rows have unequal degree"
        cols[m] = nz
    return cols


def scatter_values(mask: np.ndarray, values: np.ndarray) -> np.ndarray:
    """Dense W (zeros off the mask) from data[M][rowdeg] in canonical order."""
    cols = canonical_columns(mask)
    W = np.zeros(mask.shape, dtype=values.dtype)
    for m in range(mask.shape[0]):
        W[m, cols[m]] = values[m]
    return W


# --------------------------------------------------------------------------
# Section 5: O = W_s x I
# --------------------------------------------------------------------------
def spmm_definition(mask: np.ndarray, W: np.ndarray, I: np.ndarray) -> np.ndarray:
    """O[m][n] = sum_k mask[m][k] W[m][k] I[k][n], float64, k ascending."""
    M, K = mask.shape
    N = I.shape[1]
    O = np.zeros((M, N), dtype=np.float64)
    I64 = I.astype(np.float64)
    for m in range(M):
        for k in range(K):
            if mask[m, k]:
                O[m] += float(W[m, k]) * I64[k]
    return O


def spmm_bruteforce_scalar(mask, W, I):
    """Same sum with scalar Python loops only (tiny inputs)."""
    M, K = mask.shape
    N = I.shape[1]
    O = [[0.0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                if mask[m][k]:
                    acc += float(W[m][k]) * float(I[k][n])
            O[m][n] = acc
    return np.array(O, dtype=np.float64).reshape(M, N)


# --------------------------------------------------------------------------
# Backward products of O = W_s x I with the mask held fixed (Section 6: the
# masks are predefined and stay fixed during training).  The paper does not
# spell these out; they are the two gradients of the product by the chain rule.
# --------------------------------------------------------------------------
def transpose_order(mask: np.ndarray) -> np.ndarray:
    """perm[s] = t: the s-th kept value of W_s^T (canonical order of the
    transposed mask, i.e. row by row of mask^T, ascending column) is the t-th
    kept value of W_s (canonical order of mask)."""
    M, K = mask.shape
    index = np.full((M, K), -1, dtype=np.int64)
    t = 0
    for m in range(M):
        for k in range(K):
            if mask[m, k]:
                index[m, k] = t
                t += 1
    perm = []
    for k in range(K):
        for m in range(M):
            if mask[m, k]:
                perm.append(index[m, k])
    return np.array(perm, dtype=np.int64)


def spmm_transposed_definition(mask: np.ndarray, W: np.ndarray, dO: np.ndarray) -> np.ndarray:
    """dI[k][n] = sum_m mask[m][k] W[m][k] dO[m][n], float64 (gradient of the
    product with respect to I)."""
    M, K = mask.shape
    dI = np.zeros((K, dO.shape[1]), dtype=np.float64)
    dO64 = dO.astype(np.float64)
    for m in range(M):
        for k in range(K):
            if mask[m, k]:
                dI[k] += float(W[m, k]) * dO64[m]
    return dI


def sddmm_definition(mask: np.ndarray, dO: np.ndarray, I: np.ndarray) -> np.ndarray:
    """dW[m][t] = sum_n dO[m][n] I[k][n] for the t-th kept column k of row m,
    float64, data[M][rowdeg] in canonical order (gradient of the product with
    respect to the kept values; nothing is computed off the mask)."""
    cols = canonical_columns(mask)
    dO64, I64 = dO.astype(np.float64), I.astype(np.float64)
    dW = np.zeros(cols.shape, dtype=np.float64)
    for m in range(mask.shape[0]):
        for t, k in enumerate(cols[m]):
            dW[m, t] = float(np.sum(dO64[m] * I64[k]))
    return dW


# --------------------------------------------------------------------------
# convolution lowered to a matrix (Section 5 "GPU Implementation": the dense
# operand is the batched input activations)
# --------------------------------------------------------------------------
def im2col_3x3(X: np.ndarray) -> np.ndarray:
    """X[channel][image][H][W] -> I[9*channel + 3*(dy+1) + (dx+1)][(image*H + y)*W + x]
    = X[channel][image][y+dy][x+dx], zero outside the image (3x3 taps, stride 1,
    zero padding 1), written as explicit loops over the taps."""
    C, B, H, W = X.shape
    I = np.zeros((9 * C, B * H * W), dtype=X.dtype)
    for c in range(C):
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                k = 9 * c + 3 * (dy + 1) + (dx + 1)
                shifted = np.zeros((B, H, W), dtype=X.dtype)
                ys, ye = max(0, -dy), min(H, H - dy)
                xs, xe = max(0, -dx), min(W, W - dx)
                shifted[:, ys:ye, xs:xe] = X[c, :, ys + dy:ye + dy, xs + dx:xe + dx]
                I[k] = shifted.reshape(-1)
    return I


def col2im_3x3(Z: np.ndarray, B: int, H: int, W: int) -> np.ndarray:
    """Adjoint of im2col_3x3: Z[9*channel + 3*(dy+1) + (dx+1)][(image*H + y)*W + x] is
    added to X[channel][image][y+dy][x+dx] wherever that pixel lies inside the image
    (the gradient of the lowered input flows back to the activations)."""
    C = Z.shape[0] // 9
    X = np.zeros((C, B, H, W), dtype=np.float64)
    for c in range(C):
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                z = Z[9 * c + 3 * (dy + 1) + (dx + 1)].reshape(B, H, W)
                ys, ye = max(0, -dy), min(H, H - dy)
                xs, xe = max(0, -dx), min(W, W - dx)
                X[c, :, ys + dy:ye + dy, xs + dx:xe + dx] += z[:, ys:ye, xs:xe]
    return X


# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """IEEE float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    r = np.where(nan, (u >> 16) | 0x40, r)
    return (r & 0xFFFF).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------
# error metric of the parity tests
# --------------------------------------------------------------------------
def normalised_error(O_test: np.ndarray, O_ref: np.ndarray, denom: np.ndarray) -> float:
    """max |O_test - O_ref| / sum_k |W||I| ; where the denominator is zero the
    tested value must be exactly zero (returns inf otherwise)."""
    diff = np.abs(O_test.astype(np.float64) - O_ref)
    zero = denom == 0
    if np.any(diff[zero] != 0):
        return math.inf
    if np.all(zero):
        return 0.0
    return float(np.max(diff[~zero] / denom[~zero]))
