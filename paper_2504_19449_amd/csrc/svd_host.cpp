// Host SVD for rsparse_prepare: randomized block subspace iteration (Halko, Martinsson, Tropp,
// "Finding structure with randomness", 2011, Alg. 4.4 + 5.1) with a cyclic Jacobi eigensolver for
// the small projected problem.  Offline code: clarity over speed, threads over rows only.
#include "svd_host.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

namespace rsparse {
namespace {

template <typename F>
void par_rows(size_t n, F &&f)
{
    unsigned nt = std::thread::hardware_concurrency();
    if (nt == 0) nt = 1;
    if (nt > 16) nt = 16;
    if (n < 4 * nt) nt = 1;
    std::vector<std::thread> th;
    for (unsigned t = 0; t < nt; ++t)
        th.emplace_back([&, t]() {
            const size_t lo = n * t / nt, hi = n * (t + 1) / nt;
            for (size_t i = lo; i < hi; ++i) f(i);
        });
    for (auto &x : th) x.join();
}

double dot(const double *a, const double *b, size_t n)
{
    double s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    size_t i = 0;
    for (; i + 4 <= n; i += 4) {
        s0 += a[i] * b[i]; s1 += a[i + 1] * b[i + 1]; s2 += a[i + 2] * b[i + 2]; s3 += a[i + 3] * b[i + 3];
    }
    for (; i < n; ++i) s0 += a[i] * b[i];
    return (s0 + s1) + (s2 + s3);
}

// A block of l vectors of length len, each contiguous: v(j) = data + j*len.
struct Block {
    size_t l, len;
    std::vector<double> data;
    Block(size_t l_, size_t len_) : l(l_), len(len_), data(l_ * len_, 0.0) {}
    double *v(size_t j) { return data.data() + j * len; }
    const double *v(size_t j) const { return data.data() + j * len; }
};

// out(j)[i] = A[i,:] . in(j)  for A [rows][cols] row-major: out = A * in (as column lists).
void apply(const double *A, size_t rows, size_t cols, const Block &in, Block &out)
{
    par_rows(rows, [&](size_t i) {
        const double *a = A + i * cols;
        for (size_t j = 0; j < in.l; ++j) out.v(j)[i] = dot(a, in.v(j), cols);
    });
}

// Orthonormalise the block in place (Gram-Schmidt, each vector projected twice).
// Returns the number of vectors whose norm collapsed (rank deficiency); those are zeroed.
int orthonormalise(Block &b)
{
    int dead = 0;
    for (size_t j = 0; j < b.l; ++j) {
        double *vj = b.v(j);
        const double n0 = std::sqrt(dot(vj, vj, b.len));
        for (int pass = 0; pass < 2; ++pass) {
            std::vector<double> c(j);
            par_rows(j, [&](size_t k) { c[k] = dot(b.v(k), vj, b.len); });
            for (size_t k = 0; k < j; ++k) {
                const double *vk = b.v(k);
                const double ck = c[k];
                if (ck != 0.0)
                    for (size_t i = 0; i < b.len; ++i) vj[i] -= ck * vk[i];
            }
        }
        const double n1 = std::sqrt(dot(vj, vj, b.len));
        if (!(n1 > 1e-13 * (n0 > 0 ? n0 : 1.0))) {
            std::fill(vj, vj + b.len, 0.0);
            ++dead;
        } else {
            const double inv = 1.0 / n1;
            for (size_t i = 0; i < b.len; ++i) vj[i] *= inv;
        }
    }
    return dead;
}

// Cyclic Jacobi eigen-decomposition of the symmetric l x l matrix G (row-major, destroyed):
// eigenvalues in `w`, eigenvectors in the columns of E (row-major).  Returns sweeps used or -1.
int jacobi_eigh(std::vector<double> &G, size_t l, std::vector<double> &w, std::vector<double> &E)
{
    E.assign(l * l, 0.0);
    for (size_t i = 0; i < l; ++i) E[i * l + i] = 1.0;
    double fro = 0;
    for (double g : G) fro += g * g;
    const double tol = 1e-30 * (fro > 0 ? fro : 1.0);
    for (int sweep = 0; sweep < 60; ++sweep) {
        double off = 0;
        for (size_t p = 0; p < l; ++p)
            for (size_t q = p + 1; q < l; ++q) off += G[p * l + q] * G[p * l + q];
        if (off <= tol) {
            w.resize(l);
            for (size_t i = 0; i < l; ++i) w[i] = G[i * l + i];
            return sweep;
        }
        for (size_t p = 0; p + 1 < l; ++p)
            for (size_t q = p + 1; q < l; ++q) {
                const double apq = G[p * l + q];
                if (std::fabs(apq) < 1e-300) continue;
                const double app = G[p * l + p], aqq = G[q * l + q];
                const double theta = (aqq - app) / (2.0 * apq);
                const double t = (theta >= 0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
                const double c = 1.0 / std::sqrt(t * t + 1.0), s = t * c;
                for (size_t k = 0; k < l; ++k) {      // columns p, q
                    const double gkp = G[k * l + p], gkq = G[k * l + q];
                    G[k * l + p] = c * gkp - s * gkq;
                    G[k * l + q] = s * gkp + c * gkq;
                }
                for (size_t k = 0; k < l; ++k) {      // rows p, q
                    const double gpk = G[p * l + k], gqk = G[q * l + k];
                    G[p * l + k] = c * gpk - s * gqk;
                    G[q * l + k] = s * gpk + c * gqk;
                }
                for (size_t k = 0; k < l; ++k) {
                    const double ekp = E[k * l + p], ekq = E[k * l + q];
                    E[k * l + p] = c * ekp - s * ekq;
                    E[k * l + q] = s * ekp + c * ekq;
                }
            }
    }
    return -1;
}

uint64_t splitmix(uint64_t &s)
{
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
double gaussian(uint64_t &s)
{
    const double u1 = ((splitmix(s) >> 11) + 1.0) / 9007199254740993.0;
    const double u2 = (splitmix(s) >> 11) / 9007199254740992.0;
    return std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586 * u2);
}

}  // namespace

int svd_top_r(const double *W, int m_, int n_, int r_, double *U, double *S, double *V, char *msg, size_t msglen)
{
    const size_t m = m_, n = n_, r = r_, p = std::min(m, n);
    if (r == 0) return 0;
    if (r > p) { snprintf(msg, msglen, "rank exceeds min(m, n)"); return -1; }
    const size_t l = std::min(p, 2 * r + 16);

    std::vector<double> Wt(n * m);                 // W^T row-major, so both products are row dots
    par_rows(n, [&](size_t c) { for (size_t o = 0; o < m; ++o) Wt[c * m + o] = W[o * n + c]; });

    Block Z(l, n), Q(l, m);
    uint64_t seed = 0x5eed5eedull;
    for (double &x : Z.data) x = gaussian(seed);
    apply(W, m, n, Z, Q);
    orthonormalise(Q);

    std::vector<double> ritz(r, 0.0), prev(r, 0.0), G, w, E;
    std::vector<size_t> order(l);
    Block B(l, n);
    const int max_iter = (l == p) ? 1 : 80;
    bool converged = false;
    for (int it = 0; it < max_iter && !converged; ++it) {
        apply(Wt.data(), n, m, Q, Z);              // Z = W^T Q
        B.data = Z.data;                           // rows of B = Q^T W (before orthonormalising Z)
        // Ritz values from the projected Gram matrix G = B B^T
        G.assign(l * l, 0.0);
        par_rows(l, [&](size_t a) { for (size_t b = a; b < l; ++b) G[a * l + b] = dot(B.v(a), B.v(b), n); });
        for (size_t a = 0; a < l; ++a) for (size_t b = 0; b < a; ++b) G[a * l + b] = G[b * l + a];
        if (jacobi_eigh(G, l, w, E) < 0) { snprintf(msg, msglen, "Jacobi eigensolver did not converge"); return -1; }
        for (size_t i = 0; i < l; ++i) order[i] = i;
        std::sort(order.begin(), order.end(), [&](size_t a, size_t b) { return w[a] > w[b]; });
        double change = 0;
        for (size_t i = 0; i < r; ++i) {
            ritz[i] = std::sqrt(std::max(0.0, w[order[i]]));
            change = std::max(change, std::fabs(ritz[i] - prev[i]) / (ritz[0] > 0 ? ritz[0] : 1.0));
        }
        prev = ritz;
        if (l == p || change < 1e-10) { converged = true; break; }
        orthonormalise(Z);
        apply(W, m, n, Z, Q);                      // Q = W Z
        orthonormalise(Q);
    }
    if (!converged) { snprintf(msg, msglen, "subspace iteration did not settle in 80 iterations"); return -1; }

    // U = Q E_r,  V = B^T E_r / sigma
    for (size_t i = 0; i < r; ++i) S[i] = ritz[i];
    par_rows(m, [&](size_t o) {
        for (size_t i = 0; i < r; ++i) {
            double s = 0;
            for (size_t a = 0; a < l; ++a) s += Q.v(a)[o] * E[a * l + order[i]];
            U[o * r + i] = s;
        }
    });
    par_rows(n, [&](size_t c) {
        for (size_t i = 0; i < r; ++i) {
            double s = 0;
            for (size_t a = 0; a < l; ++a) s += B.v(a)[c] * E[a * l + order[i]];
            V[c * r + i] = S[i] > 0 ? s / S[i] : 0.0;
        }
    });
    return 0;
}

}  // namespace rsparse
