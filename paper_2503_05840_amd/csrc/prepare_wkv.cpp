// Offline weight transform of slim attention (eq. 6 of the paper): W_KV = W_K^{-1} W_V.
//
// Host only, fp64 throughout (App. A converts to fp64 "for better accuracy of matrix
// inversion").  Instead of forming the inverse and multiplying, the d right-hand sides of
// W_K W_KV = W_V are solved with one blocked LU factorisation with partial pivoting; the
// acceptance check of App. A (W_K W_KV close to W_V) is the same for both routes.
//
// Blocked right-looking LU on the augmented rows [A | B]: per panel of NB columns, an
// unblocked pivoted factorisation, a unit-lower triangular solve for the panel's row block,
// and a rank-NB update of everything below, threaded over row strips.  Back substitution is
// blocked the same way.  A 1-norm condition estimate (Hager's iteration on the LU factors)
// is returned for the caller's sanity check.
#include "slim_attention.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

namespace {

constexpr int NB = 64;        // panel width
constexpr int CB = 256;       // column chunk kept in L1 during a rank-NB update

int host_threads() {
  unsigned n = std::thread::hardware_concurrency();
  if (n == 0) n = 1;
  return (int)std::min(n, 32u);
}

template <class F>
void parallel_rows(int lo, int hi, int grain, F&& body) {
  int n = hi - lo;
  if (n <= 0) return;
  int nt = std::min(host_threads(), std::max(1, n / grain));
  if (nt <= 1) { body(lo, hi); return; }
  std::vector<std::thread> th;
  int per = (n + nt - 1) / nt;
  per = (per + 3) & ~3;
  for (int t = 0; t < nt; ++t) {
    int a = lo + t * per, b = std::min(hi, a + per);
    if (a >= b) break;
    th.emplace_back([=, &body] { body(a, b); });
  }
  for (auto& x : th) x.join();
}

// C[i][0..n) -= sum_kk Acol[i][kk] * R[kk][0..n)   for i in [r0, r1)
//   C  : row pitch ldc;  Acol: element (i, kk) at A[i*lda + kk];  R: row pitch ldr, kb rows
void rank_update(double* C, long ldc, const double* A, long lda, const double* R, long ldr,
                 int r0, int r1, int kb, int n) {
  for (int c0 = 0; c0 < n; c0 += CB) {
    int cw = std::min(CB, n - c0);
    int i = r0;
    for (; i + 4 <= r1; i += 4) {
      double* c0p = C + (long)(i + 0) * ldc + c0;
      double* c1p = C + (long)(i + 1) * ldc + c0;
      double* c2p = C + (long)(i + 2) * ldc + c0;
      double* c3p = C + (long)(i + 3) * ldc + c0;
      for (int kk = 0; kk < kb; ++kk) {
        const double a0 = A[(long)(i + 0) * lda + kk], a1 = A[(long)(i + 1) * lda + kk];
        const double a2 = A[(long)(i + 2) * lda + kk], a3 = A[(long)(i + 3) * lda + kk];
        const double* r = R + (long)kk * ldr + c0;
        for (int c = 0; c < cw; ++c) {
          const double rv = r[c];
          c0p[c] -= a0 * rv; c1p[c] -= a1 * rv; c2p[c] -= a2 * rv; c3p[c] -= a3 * rv;
        }
      }
    }
    for (; i < r1; ++i) {
      double* cp = C + (long)i * ldc + c0;
      for (int kk = 0; kk < kb; ++kk) {
        const double a = A[(long)i * lda + kk];
        const double* r = R + (long)kk * ldr + c0;
        for (int c = 0; c < cw; ++c) cp[c] -= a * r[c];
      }
    }
  }
}

struct LU {
  int d;
  std::vector<double> a;     // factors: unit L below the diagonal, U on and above
  std::vector<int> perm;     // row i of the factored matrix is row perm[i] of W_K
};

// x := A^{-1} x  using P A = L U
void solve_vec(const LU& f, std::vector<double>& x) {
  const int d = f.d;
  std::vector<double> y(d);
  for (int i = 0; i < d; ++i) y[i] = x[f.perm[i]];
  for (int i = 0; i < d; ++i) {
    const double* row = &f.a[(long)i * d];
    double s = y[i];
    for (int j = 0; j < i; ++j) s -= row[j] * y[j];
    y[i] = s;
  }
  for (int i = d - 1; i >= 0; --i) {
    const double* row = &f.a[(long)i * d];
    double s = y[i];
    for (int j = i + 1; j < d; ++j) s -= row[j] * y[j];
    y[i] = s / row[i];
  }
  x.swap(y);
}

// x := A^{-T} x :  A^T = U^T L^T P
void solve_vec_transposed(const LU& f, std::vector<double>& x) {
  const int d = f.d;
  std::vector<double> w(x);
  for (int i = 0; i < d; ++i) {            // U^T w = x  (forward, column-oriented on rows of U)
    const double* row = &f.a[(long)i * d];
    w[i] /= row[i];
    const double wi = w[i];
    for (int j = i + 1; j < d; ++j) w[j] -= row[j] * wi;
  }
  for (int i = d - 1; i >= 0; --i) {       // L^T v = w  (backward)
    const double* row = &f.a[(long)i * d];
    const double wi = w[i];
    for (int j = 0; j < i; ++j) w[j] -= row[j] * wi;
  }
  for (int i = 0; i < d; ++i) x[f.perm[i]] = w[i];
}

double inverse_one_norm_estimate(const LU& f) {
  const int d = f.d;
  std::vector<double> x(d, 1.0 / d), z(d);
  double est = 0.0;
  for (int it = 0; it < 5; ++it) {
    solve_vec(f, x);
    double n1 = 0.0;
    for (double v : x) n1 += std::fabs(v);
    if (it > 0 && n1 <= est) break;
    est = n1;
    for (int i = 0; i < d; ++i) z[i] = x[i] >= 0 ? 1.0 : -1.0;
    solve_vec_transposed(f, z);
    int jmax = 0;
    for (int i = 1; i < d; ++i) if (std::fabs(z[i]) > std::fabs(z[jmax])) jmax = i;
    std::fill(x.begin(), x.end(), 0.0);
    x[jmax] = 1.0;
  }
  return est;
}

}  // namespace

namespace {

// X = A^{-1} B for A (d x d) and B, X (d x nr), row-major; see the header comment of this file.
int lu_solve(const double* Wk, const double* Wv, double* Wkv, int d, int nr, double* rcond_out) {
  const long dd = (long)d * d, dn = (long)d * nr;

  LU f;
  f.d = d;
  f.a.assign(Wk, Wk + dd);
  f.perm.resize(d);
  for (int i = 0; i < d; ++i) f.perm[i] = i;
  std::vector<double> b(Wv, Wv + dn);

  double amax = 0.0, anorm1 = 0.0;
  {
    std::vector<double> colsum(d, 0.0);
    for (long i = 0; i < dd; ++i) {
      const double v = f.a[i];
      if (!std::isfinite(v)) return SLIM_ERR_SINGULAR;
      amax = std::max(amax, std::fabs(v));
      colsum[i % d] += std::fabs(v);
    }
    for (long i = 0; i < dn; ++i)
      if (!std::isfinite(b[i])) return SLIM_ERR_SINGULAR;
    for (double s : colsum) anorm1 = std::max(anorm1, s);
  }
  const double tiny = 2.220446049250313e-16 * d * amax;
  double* A = f.a.data();
  double* Bm = b.data();

  for (int k0 = 0; k0 < d; k0 += NB) {
    const int kb = std::min(NB, d - k0);
    const int k1 = k0 + kb;
    // --- panel: columns [k0, k1), rows [k0, d), unblocked with partial pivoting -------------
    for (int j = k0; j < k1; ++j) {
      int p = j;
      double best = std::fabs(A[(long)j * d + j]);
      for (int i = j + 1; i < d; ++i) {
        const double v = std::fabs(A[(long)i * d + j]);
        if (v > best) { best = v; p = i; }
      }
      if (!(best > tiny)) return SLIM_ERR_SINGULAR;
      if (p != j) {
        std::swap_ranges(A + (long)j * d, A + (long)j * d + d, A + (long)p * d);
        std::swap_ranges(Bm + (long)j * nr, Bm + (long)j * nr + nr, Bm + (long)p * nr);
        std::swap(f.perm[j], f.perm[p]);
      }
      const double inv = 1.0 / A[(long)j * d + j];
      const double* prow = A + (long)j * d;
      parallel_rows(j + 1, d, 512, [&](int a, int e) {
        for (int i = a; i < e; ++i) {
          double* row = A + (long)i * d;
          const double l = row[j] * inv;
          row[j] = l;
          for (int c = j + 1; c < k1; ++c) row[c] -= l * prow[c];
        }
      });
    }
    // --- row block: [A12 | B1] := L11^{-1} [A12 | B1]  (unit lower, rows k0..k1) ------------
    for (int i = k0 + 1; i < k1; ++i) {
      double* arow = A + (long)i * d;
      double* brow = Bm + (long)i * nr;
      for (int j = k0; j < i; ++j) {
        const double l = arow[j];
        const double* ar = A + (long)j * d;
        const double* br = Bm + (long)j * nr;
        for (int c = k1; c < d; ++c) arow[c] -= l * ar[c];
        for (int c = 0; c < nr; ++c) brow[c] -= l * br[c];
      }
    }
    // --- trailing update: A22 -= A21 A12 ; B2 -= A21 B1 --------------------------------------
    parallel_rows(k1, d, 16, [&](int a, int e) {
      if (d - k1 > 0)
        rank_update(A + k1, d, A + k0, d, A + (long)k0 * d + k1, d, a, e, kb, d - k1);
      rank_update(Bm, nr, A + k0, d, Bm + (long)k0 * nr, nr, a, e, kb, nr);
    });
  }

  // --- back substitution: U X = Y, blocked from the bottom ------------------------------------
  for (int k1 = d; k1 > 0; k1 -= NB) {
    const int k0 = std::max(0, k1 - NB);
    const int kb = k1 - k0;
    for (int j = k1 - 1; j >= k0; --j) {
      double* brow = Bm + (long)j * nr;
      const double inv = 1.0 / A[(long)j * d + j];
      for (int c = 0; c < nr; ++c) brow[c] *= inv;
      for (int i = k0; i < j; ++i) {
        const double u = A[(long)i * d + j];
        double* bi = Bm + (long)i * nr;
        for (int c = 0; c < nr; ++c) bi[c] -= u * brow[c];
      }
    }
    parallel_rows(0, k0, 16, [&](int a, int e) {
      rank_update(Bm, nr, A + k0, d, Bm + (long)k0 * nr, nr, a, e, kb, nr);
    });
  }
  std::memcpy(Wkv, Bm, sizeof(double) * dn);

  const double inv_norm = inverse_one_norm_estimate(f);
  const double rcond = (anorm1 > 0 && inv_norm > 0) ? 1.0 / (anorm1 * inv_norm) : 0.0;
  if (rcond_out) *rcond_out = rcond;
  return rcond < 1e-12 ? SLIM_ERR_ILLCOND : SLIM_OK;
}

}  // namespace

extern "C" int slim_prepare_wkv(const double* Wk, const double* Wv, double* Wkv, int d,
                                double* rcond_out) {
  if (!Wk || !Wv || !Wkv) return SLIM_ERR_ARG;
  if (d < 1) return SLIM_ERR_SHAPE;
  return lu_solve(Wk, Wv, Wkv, d, d, rcond_out);
}

// Non-square projections, option 1: W_K is d x e with e > d and has no inverse, but the right
// inverse W_K^T (W_K W_K^T)^{-1} gives W_KV = W_K^T (W_K W_K^T)^{-1} W_V (e x e) with
// (X W_K) W_KV = X W_V exactly.  G = W_K W_K^T is formed in fp64, G Z = W_V is solved with the same
// LU (d x e right-hand sides), and W_KV = W_K^T Z.
extern "C" int slim_prepare_wkv_nonsquare(const double* Wk, const double* Wv, double* Wkv, int d, int e,
                                          double* rcond_out) {
  if (!Wk || !Wv || !Wkv) return SLIM_ERR_ARG;
  if (d < 1 || e < d) return SLIM_ERR_SHAPE;
  std::vector<double> G((size_t)d * d), Z((size_t)d * e);
  parallel_rows(0, d, 8, [&](int a, int b) {
    for (int i = a; i < b; ++i)
      for (int j = 0; j <= i; ++j) {
        const double* ri = Wk + (size_t)i * e;
        const double* rj = Wk + (size_t)j * e;
        double s = 0.0;
        for (int c = 0; c < e; ++c) s += ri[c] * rj[c];
        G[(size_t)i * d + j] = s;
      }
  });
  for (int i = 0; i < d; ++i)
    for (int j = i + 1; j < d; ++j) G[(size_t)i * d + j] = G[(size_t)j * d + i];
  const int rc = lu_solve(G.data(), Wv, Z.data(), d, e, rcond_out);
  if (rc != SLIM_OK && rc != SLIM_ERR_ILLCOND) return rc;
  parallel_rows(0, e, 8, [&](int a, int b) {
    for (int i = a; i < b; ++i) {                       // row i of W_KV = sum_k W_K[k][i] Z[k][:]
      double* out = Wkv + (size_t)i * e;
      for (int c = 0; c < e; ++c) out[c] = 0.0;
      for (int k = 0; k < d; ++k) {
        const double w = Wk[(size_t)k * e + i];
        const double* z = Z.data() + (size_t)k * e;
        for (int c = 0; c < e; ++c) out[c] += w * z[c];
      }
    }
  });
  return rc;
}

extern "C" int slim_pack_weights(const double* W, void* dst_host, int rows, int cols, int dtype) {
  if (!W || !dst_host) return SLIM_ERR_ARG;
  if (rows < 1 || cols < 1) return SLIM_ERR_SHAPE;
  const long n = (long)rows * cols;
  if (dtype == SLIM_F32) {
    float* o = (float*)dst_host;
    for (long i = 0; i < n; ++i) o[i] = (float)W[i];
    return SLIM_OK;
  }
  if (dtype == SLIM_BF16) {
    uint16_t* o = (uint16_t*)dst_host;
    for (long i = 0; i < n; ++i) {
      const float f = (float)W[i];
      uint32_t u;
      std::memcpy(&u, &f, 4);
      if ((u & 0x7fffffffu) > 0x7f800000u) { o[i] = (uint16_t)((u >> 16) | 0x40); continue; }  // NaN
      u += 0x7fffu + ((u >> 16) & 1u);                                                         // RNE
      o[i] = (uint16_t)(u >> 16);
    }
    return SLIM_OK;
  }
  return SLIM_ERR_DTYPE;
}

extern "C" int slim_band_kcache(const void* src_host, void* dst_host, int B, int64_t t_stride, int H, int d_k,
                                int elem_bytes) {
  if (!src_host || !dst_host) return SLIM_ERR_ARG;
  if (B < 1 || t_stride < 1 || H < 1 || d_k < 1 || (elem_bytes != 2 && elem_bytes != 4)) return SLIM_ERR_SHAPE;
  if (t_stride % 32 != 0) return SLIM_ERR_LAYOUT;
  const size_t row = (size_t)H * d_k * elem_bytes, piece = (size_t)d_k * elem_bytes;
  const char* src = (const char*)src_host;
  char* dst = (char*)dst_host;
  for (int64_t r = 0; r < (int64_t)B * t_stride; ++r) {      // bands never straddle sequences: t_stride % 32 == 0
    const size_t band = (size_t)(r / 32), rin = (size_t)(r % 32);
    for (int h = 0; h < H; ++h)
      std::memcpy(dst + ((band * H + h) * 32 + rin) * piece, src + (size_t)r * row + (size_t)h * piece, piece);
  }
  return SLIM_OK;
}

// RoPE appendix: the one table both rotation directions use.
extern "C" int slim_rope_table(float* table_host, int T, int d_k, double base) {
  if (!table_host) return SLIM_ERR_ARG;
  if (T < 1 || d_k < 2 || (d_k & 1) || !(base > 0.0)) return SLIM_ERR_SHAPE;
  const int half = d_k / 2;
  for (int j = 0; j < half; ++j) {
    const double theta = std::pow(base, -2.0 * (double)j / (double)d_k);
    for (long t = 0; t < T; ++t) {
      const double ang = (double)t * theta;
      table_host[((size_t)t * half + j) * 2 + 0] = (float)std::cos(ang);
      table_host[((size_t)t * half + j) * 2 + 1] = (float)std::sin(ang);
    }
  }
  return SLIM_OK;
}
