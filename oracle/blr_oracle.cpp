// CPU oracle for the block low-rank (BLR) linear forward pass: Monarch, BLAST, low-rank, dense.
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. It exists so that the GPU
// library can be checked against an independent, slow, obviously-correct
// implementation. Only the tests, the smoke check and the benchmark's
// cpu_baseline leg may call it. It shares no code with the GPU path.
//
// Everything is fp64, row-major, host memory. Inputs are the exact values the
// GPU sees (already rounded to the storage type by the input generator); no
// intermediate is ever rounded. Each operator is evaluated factor by factor in
// the order the paper states (Section 2.1 "Weight Structures", and the layout
// statement in Section 4 "Monarch", optimisation 1), with every intermediate
// tensor written out in full so a reader can follow it by eye. A second form
// materialises the dense weight from the per-block definitions and multiplies
// by brute force.
//
// Notation (paper -> here). The paper writes Y = X W with W in R^{i x o}; the
// library boundary uses W[n_out][n_in] and Y = X W^T. Tokens n -> T, features
// i, o -> n_in, n_out. Monarch: b1 = b2 = b = nblocks, p = n_in/b, q = n_out/b,
// per-block rank r' = r/b; the paper's stored tensors V (b1, r' b2, p) and
// U (b2, q, b1 r') are called R and L here. BLAST: input block j (paper l),
// output block i (paper k); V[b][n_in/b][r], S[i][j][r], U[b][n_out/b][r]
// (the paper's U_k in R^{r x q} is stored transposed).
//
// Parity pins for every function in this file live in tests/test_oracle_*.py.

#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>
#include <algorithm>

namespace {

template <class F>
void parallel_over_tokens(int64_t T, int nthreads, F&& body) {
    if (nthreads < 1) nthreads = 1;
    if ((int64_t)nthreads > T) nthreads = (int)std::max<int64_t>(T, 1);
    if (nthreads == 1) { body(0, T, 0); return; }
    std::vector<std::thread> pool;
    int64_t chunk = (T + nthreads - 1) / nthreads;
    for (int w = 0; w < nthreads; ++w) {
        int64_t t0 = w * chunk, t1 = std::min<int64_t>(T, t0 + chunk);
        if (t0 >= t1) break;
        pool.emplace_back([=, &body] { body(t0, t1, w); });
    }
    for (auto& th : pool) th.join();
}

}  // namespace

extern "C" {

enum { BLR_ORACLE_OUT_INTERLEAVED = 0, BLR_ORACLE_OUT_BLOCKED = 1 };

// ---------------------------------------------------------------------------
// Dense: Y = X W^T (Section 2.1, "Dense"), brute force.
// X[T][n_in], W[n_out][n_in], Y[T][n_out].
// ---------------------------------------------------------------------------
int blr_oracle_dense_forward(const double* X, const double* W, double* Y,
                             int64_t T, int n_in, int n_out, int nthreads) {
    if (!X || !W || !Y || T < 0 || n_in <= 0 || n_out <= 0) return 1;
    parallel_over_tokens(T, nthreads, [&](int64_t t0, int64_t t1, int) {
        for (int64_t t = t0; t < t1; ++t)
            for (int o = 0; o < n_out; ++o) {
                double acc = 0.0;
                for (int a = 0; a < n_in; ++a) acc += X[t * n_in + a] * W[(int64_t)o * n_in + a];
                Y[t * n_out + o] = acc;
            }
    });
    return 0;
}

// ---------------------------------------------------------------------------
// The middle permutation of a Monarch layer (Section 2.1, Fig. 2 left,
// "b1 <=> b2"; Section 4 optimisation 1 for the two storage orders).
//
// After the first batched product the middle vector of one token is
// z[l][c], l = input block, c in [0, r), and the first factor stores its rows
// with the output-block index k fastest: c = rho*b + k. The second factor
// expects z'[k][m] with m = l*r' + rho (rho fastest, then l). Written flat on
// the b*r middle vector: dst index k*r + l*r' + rho  <-  src index l*r + rho*b + k.
// perm[dst] = src.
// ---------------------------------------------------------------------------
int blr_oracle_monarch_middle_perm(int nblocks, int r, int64_t* perm) {
    if (!perm || nblocks <= 0 || r <= 0 || r % nblocks) return 1;
    const int b = nblocks, rp = r / b;
    for (int k = 0; k < b; ++k)
        for (int l = 0; l < b; ++l)
            for (int rho = 0; rho < rp; ++rho)
                perm[(int64_t)k * r + l * rp + rho] = (int64_t)l * r + rho * b + k;
    return 0;
}

// ---------------------------------------------------------------------------
// Monarch forward, factor by factor (Section 2.1 "Monarch": bmm, permutation,
// bmm; Section 4 optimisation 3 for the order of the output features).
//   1. Z[t][l][c]   = sum_a X[t][l*p + a] * R[l][c][a]
//   2. Z'[t][k][m]  = Z[t][l][rho*b + k],   m = l*r' + rho
//   3. Yb[t][k][j]  = sum_m Z'[t][k][m] * L[k][j][m]
//   4. interleaved: Y[t][j*b + k] = Yb[t][k][j]   (the (n, q, b2) order)
//      blocked:     Y[t][k*q + j] = Yb[t][k][j]   (the (n, b2, q) order)
// R[b][r][p], L[b][q][r]. macs (optional) receives the multiply-adds executed.
// ---------------------------------------------------------------------------
int blr_oracle_monarch_forward(const double* X, const double* R, const double* L, double* Y,
                               int64_t T, int n_in, int n_out, int nblocks, int r,
                               int out_order, int nthreads, int64_t* macs) {
    if (!X || !R || !L || !Y || T < 0 || n_in <= 0 || n_out <= 0 || nblocks <= 0 || r <= 0) return 1;
    if (n_in % nblocks || n_out % nblocks || r % nblocks) return 1;
    if (out_order != BLR_ORACLE_OUT_INTERLEAVED && out_order != BLR_ORACLE_OUT_BLOCKED) return 1;
    const int b = nblocks, p = n_in / b, q = n_out / b, rp = r / b;
    std::vector<int64_t> counts(std::max(nthreads, 1) + 1, 0);
    parallel_over_tokens(T, nthreads, [&](int64_t t0, int64_t t1, int w) {
        std::vector<double> Z((size_t)b * r), Zp((size_t)b * r), Yb((size_t)b * q);
        int64_t n = 0;
        for (int64_t t = t0; t < t1; ++t) {
            const double* x = X + t * n_in;
            for (int l = 0; l < b; ++l)
                for (int c = 0; c < r; ++c) {
                    const double* row = R + ((int64_t)l * r + c) * p;
                    double acc = 0.0;
                    for (int a = 0; a < p; ++a) acc += x[l * p + a] * row[a];
                    Z[(size_t)l * r + c] = acc;
                    n += p;
                }
            for (int k = 0; k < b; ++k)
                for (int l = 0; l < b; ++l)
                    for (int rho = 0; rho < rp; ++rho)
                        Zp[(size_t)k * r + l * rp + rho] = Z[(size_t)l * r + rho * b + k];
            for (int k = 0; k < b; ++k)
                for (int j = 0; j < q; ++j) {
                    const double* row = L + ((int64_t)k * q + j) * r;
                    double acc = 0.0;
                    for (int m = 0; m < r; ++m) acc += Zp[(size_t)k * r + m] * row[m];
                    Yb[(size_t)k * q + j] = acc;
                    n += r;
                }
            double* y = Y + t * n_out;
            for (int k = 0; k < b; ++k)
                for (int j = 0; j < q; ++j) {
                    int o = (out_order == BLR_ORACLE_OUT_INTERLEAVED) ? j * b + k : k * q + j;
                    y[o] = Yb[(size_t)k * q + j];
                }
        }
        counts[w] = n;
    });
    if (macs) { int64_t s = 0; for (auto c : counts) s += c; *macs = s; }
    return 0;
}

// ---------------------------------------------------------------------------
// Dense weight a Monarch layer stands for, built from the per-block
// definition W_{l,k} = V_{l,k} U_{l,k} (Section 2.1 "Monarch"), where
//   V_{l,k}[a][rho] = R[l][rho*b + k][a]      (p x r')
//   U_{l,k}[rho][j] = L[k][j][l*r' + rho]     (r' x q)
// are the slices the two storage orders of Section 4 (optimisation 1) select.
// Output W[n_out][n_in] so that Y = X W^T; row index follows out_order.
// ---------------------------------------------------------------------------
int blr_oracle_materialize_monarch(const double* R, const double* L, double* W,
                                   int n_in, int n_out, int nblocks, int r, int out_order) {
    if (!R || !L || !W || n_in <= 0 || n_out <= 0 || nblocks <= 0 || r <= 0) return 1;
    if (n_in % nblocks || n_out % nblocks || r % nblocks) return 1;
    const int b = nblocks, p = n_in / b, q = n_out / b, rp = r / b;
    for (int k = 0; k < b; ++k)
        for (int j = 0; j < q; ++j) {
            int o = (out_order == BLR_ORACLE_OUT_INTERLEAVED) ? j * b + k : k * q + j;
            for (int l = 0; l < b; ++l)
                for (int a = 0; a < p; ++a) {
                    double acc = 0.0;
                    for (int rho = 0; rho < rp; ++rho)
                        acc += R[((int64_t)l * r + rho * b + k) * p + a] *
                               L[((int64_t)k * q + j) * r + l * rp + rho];
                    W[(int64_t)o * n_in + l * p + a] = acc;
                }
        }
    return 0;
}

// ---------------------------------------------------------------------------
// Monarch with different block counts on the two sides (Section 2.1 "Monarch":
// b2 x b1 blocks, l in [0, b1) input blocks of p = n_in/b1 features, k in
// [0, b2) output blocks of q = n_out/b2 features, per-block rank r').
// Stored factors follow the same two orders as the square case:
//   R[b1][r'*b2][p], middle index rho*b2 + k;  L[b2][q][b1*r'], innermost l*r' + rho.
//   1. Z[t][l][c]    = sum_a X[t][l*p + a] * R[l][c][a],          c < r'*b2
//   2. Z'[t][k][m]   = Z[t][l][rho*b2 + k],   m = l*r' + rho      (b1 <=> b2)
//   3. Yb[t][k][j]   = sum_m Z'[t][k][m] * L[k][j][m],            m < b1*r'
//   4. interleaved: Y[t][j*b2 + k];  blocked: Y[t][k*q + j]
// ---------------------------------------------------------------------------
int blr_oracle_monarch_rect_forward(const double* X, const double* R, const double* L, double* Y,
                                    int64_t T, int n_in, int n_out, int b1, int b2, int rp,
                                    int out_order, int nthreads, int64_t* macs) {
    if (!X || !R || !L || !Y || T < 0 || n_in <= 0 || n_out <= 0 || b1 <= 0 || b2 <= 0 || rp <= 0) return 1;
    if (n_in % b1 || n_out % b2) return 1;
    if (out_order != BLR_ORACLE_OUT_INTERLEAVED && out_order != BLR_ORACLE_OUT_BLOCKED) return 1;
    const int p = n_in / b1, q = n_out / b2, w1 = rp * b2, w2 = b1 * rp;
    std::vector<int64_t> counts(std::max(nthreads, 1) + 1, 0);
    parallel_over_tokens(T, nthreads, [&](int64_t t0, int64_t t1, int w) {
        std::vector<double> Z((size_t)b1 * w1), Zp((size_t)b2 * w2), Yb((size_t)b2 * q);
        int64_t n = 0;
        for (int64_t t = t0; t < t1; ++t) {
            const double* x = X + t * n_in;
            for (int l = 0; l < b1; ++l)
                for (int c = 0; c < w1; ++c) {
                    const double* row = R + ((int64_t)l * w1 + c) * p;
                    double acc = 0.0;
                    for (int a = 0; a < p; ++a) acc += x[l * p + a] * row[a];
                    Z[(size_t)l * w1 + c] = acc;
                    n += p;
                }
            for (int k = 0; k < b2; ++k)
                for (int l = 0; l < b1; ++l)
                    for (int rho = 0; rho < rp; ++rho)
                        Zp[(size_t)k * w2 + l * rp + rho] = Z[(size_t)l * w1 + rho * b2 + k];
            for (int k = 0; k < b2; ++k)
                for (int j = 0; j < q; ++j) {
                    const double* row = L + ((int64_t)k * q + j) * w2;
                    double acc = 0.0;
                    for (int m = 0; m < w2; ++m) acc += Zp[(size_t)k * w2 + m] * row[m];
                    Yb[(size_t)k * q + j] = acc;
                    n += w2;
                }
            double* y = Y + t * n_out;
            for (int k = 0; k < b2; ++k)
                for (int j = 0; j < q; ++j)
                    y[(out_order == BLR_ORACLE_OUT_INTERLEAVED) ? j * b2 + k : k * q + j] = Yb[(size_t)k * q + j];
        }
        counts[w] = n;
    });
    if (macs) { int64_t s = 0; for (auto c : counts) s += c; *macs = s; }
    return 0;
}

// ---------------------------------------------------------------------------
// BLAST forward, factor by factor (Section 2.1 "BLAST":
// Y_k = (sum_l (X_l V_l) S_{l,k}) U_k with S diagonal), q = n_in/b, p = n_out/b.
//   1. Z[t][j][rho] = sum_c X[t][j*q + c] * V[j][c][rho]
//   2. A[t][i][rho] = sum_j S[i][j][rho] * Z[t][j][rho]
//   3. Y[t][i*p + a] = sum_rho A[t][i][rho] * U[i][a][rho]
// ---------------------------------------------------------------------------
int blr_oracle_blast_forward(const double* X, const double* U, const double* S, const double* V,
                             double* Y, int64_t T, int n_in, int n_out, int b, int r,
                             int nthreads, int64_t* macs) {
    if (!X || !U || !S || !V || !Y || T < 0 || n_in <= 0 || n_out <= 0 || b <= 0 || r <= 0) return 1;
    if (n_in % b || n_out % b) return 1;
    const int q = n_in / b, p = n_out / b;
    std::vector<int64_t> counts(std::max(nthreads, 1) + 1, 0);
    parallel_over_tokens(T, nthreads, [&](int64_t t0, int64_t t1, int w) {
        std::vector<double> Z((size_t)b * r), A((size_t)b * r);
        int64_t n = 0;
        for (int64_t t = t0; t < t1; ++t) {
            const double* x = X + t * n_in;
            for (int j = 0; j < b; ++j) {
                double* z = Z.data() + (size_t)j * r;
                for (int rho = 0; rho < r; ++rho) z[rho] = 0.0;
                for (int c = 0; c < q; ++c) {
                    const double xv = x[j * q + c];
                    const double* vrow = V + ((int64_t)j * q + c) * r;
                    for (int rho = 0; rho < r; ++rho) z[rho] += xv * vrow[rho];
                    n += r;
                }
            }
            for (int i = 0; i < b; ++i) {
                double* a = A.data() + (size_t)i * r;
                for (int rho = 0; rho < r; ++rho) a[rho] = 0.0;
                for (int j = 0; j < b; ++j) {
                    const double* s = S + ((int64_t)i * b + j) * r;
                    const double* z = Z.data() + (size_t)j * r;
                    for (int rho = 0; rho < r; ++rho) a[rho] += s[rho] * z[rho];
                    n += r;
                }
            }
            double* y = Y + t * n_out;
            for (int i = 0; i < b; ++i)
                for (int a = 0; a < p; ++a) {
                    const double* urow = U + ((int64_t)i * p + a) * r;
                    const double* av = A.data() + (size_t)i * r;
                    double acc = 0.0;
                    for (int rho = 0; rho < r; ++rho) acc += av[rho] * urow[rho];
                    y[i * p + a] = acc;
                    n += r;
                }
        }
        counts[w] = n;
    });
    if (macs) { int64_t s = 0; for (auto c : counts) s += c; *macs = s; }
    return 0;
}

// ---------------------------------------------------------------------------
// Dense weight a BLAST layer stands for: block (i, j) of W[n_out][n_in] is
// U_i diag(S[i][j]) V_j^T (Section 2.1 "BLAST", W_{l,k} = V_l S_{l,k} U_k,
// transposed to the out x in orientation).
// ---------------------------------------------------------------------------
int blr_oracle_materialize_blast(const double* U, const double* S, const double* V, double* W,
                                 int n_in, int n_out, int b, int r) {
    if (!U || !S || !V || !W || n_in <= 0 || n_out <= 0 || b <= 0 || r <= 0) return 1;
    if (n_in % b || n_out % b) return 1;
    const int q = n_in / b, p = n_out / b;
    for (int i = 0; i < b; ++i)
        for (int a = 0; a < p; ++a)
            for (int j = 0; j < b; ++j)
                for (int c = 0; c < q; ++c) {
                    double acc = 0.0;
                    for (int rho = 0; rho < r; ++rho)
                        acc += U[((int64_t)i * p + a) * r + rho] * S[((int64_t)i * b + j) * r + rho] *
                               V[((int64_t)j * q + c) * r + rho];
                    W[((int64_t)i * p + a) * n_in + j * q + c] = acc;
                }
    return 0;
}

// ---------------------------------------------------------------------------
// Low-rank forward (Section 2.1 "Low-Rank (LR)": W = V U, Y = (X V) U, with
// V in R^{i x r}, U in R^{r x o}). Both factors are stored with their
// contraction index contiguous: V[r][n_in] (the paper's V transposed) and
// U[n_out][r] (the paper's U transposed).
//   1. Z[t][c] = sum_a X[t][a] * V[c][a]
//   2. Y[t][o] = sum_c Z[t][c] * U[o][c]
// ---------------------------------------------------------------------------
int blr_oracle_lowrank_forward(const double* X, const double* V, const double* U, double* Y,
                               int64_t T, int n_in, int n_out, int r, int nthreads, int64_t* macs) {
    if (!X || !V || !U || !Y || T < 0 || n_in <= 0 || n_out <= 0 || r <= 0) return 1;
    std::vector<int64_t> counts(std::max(nthreads, 1) + 1, 0);
    parallel_over_tokens(T, nthreads, [&](int64_t t0, int64_t t1, int w) {
        std::vector<double> Z((size_t)r);
        int64_t n = 0;
        for (int64_t t = t0; t < t1; ++t) {
            const double* x = X + t * n_in;
            for (int c = 0; c < r; ++c) {
                const double* vrow = V + (int64_t)c * n_in;
                double acc = 0.0;
                for (int a = 0; a < n_in; ++a) acc += x[a] * vrow[a];
                Z[c] = acc;
                n += n_in;
            }
            double* y = Y + t * n_out;
            for (int o = 0; o < n_out; ++o) {
                const double* urow = U + (int64_t)o * r;
                double acc = 0.0;
                for (int c = 0; c < r; ++c) acc += Z[c] * urow[c];
                y[o] = acc;
                n += r;
            }
        }
        counts[w] = n;
    });
    if (macs) { int64_t s = 0; for (auto c : counts) s += c; *macs = s; }
    return 0;
}

// Dense weight a low-rank layer stands for: W[o][a] = sum_c U[o][c] V[c][a]
// (Section 2.1 "Low-Rank (LR)", W = V U in the out x in orientation).
int blr_oracle_materialize_lowrank(const double* V, const double* U, double* W, int n_in, int n_out, int r) {
    if (!V || !U || !W || n_in <= 0 || n_out <= 0 || r <= 0) return 1;
    for (int o = 0; o < n_out; ++o)
        for (int a = 0; a < n_in; ++a) {
            double acc = 0.0;
            for (int c = 0; c < r; ++c) acc += U[(int64_t)o * r + c] * V[(int64_t)c * n_in + a];
            W[(int64_t)o * n_in + a] = acc;
        }
    return 0;
}

}  // extern "C"
