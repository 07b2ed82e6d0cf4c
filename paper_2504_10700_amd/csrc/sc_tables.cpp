// Host-side coupling tables (see sc_tables.h).  Pure C++17, no HIP.
#include "sc_tables.h"

#include <algorithm>
#include <cmath>
#include <complex>
#include <map>
#include <tuple>

namespace sc {
namespace {

double factorial(int n) {
  double f = 1.0;
  for (int i = 2; i <= n; ++i) f *= i;
  return f;  // exact in double for n <= 22; callers stay below 20
}

// Wigner 3j symbol for integer angular momenta (Racah's single-sum formula).
double wigner_3j(int j1, int j2, int j3, int m1, int m2, int m3) {
  if (m1 + m2 + m3 != 0) return 0.0;
  if (j3 < std::abs(j1 - j2) || j3 > j1 + j2) return 0.0;
  if (std::abs(m1) > j1 || std::abs(m2) > j2 || std::abs(m3) > j3) return 0.0;
  const double delta = factorial(j1 + j2 - j3) * factorial(j1 - j2 + j3) * factorial(-j1 + j2 + j3) /
                       factorial(j1 + j2 + j3 + 1);
  const double pref = std::sqrt(delta * factorial(j1 + m1) * factorial(j1 - m1) * factorial(j2 + m2) *
                                factorial(j2 - m2) * factorial(j3 + m3) * factorial(j3 - m3));
  const int kmin = std::max({0, j2 - j3 - m1, j1 - j3 + m2});
  const int kmax = std::min({j1 + j2 - j3, j1 - m1, j2 + m2});
  double sum = 0.0;
  for (int k = kmin; k <= kmax; ++k) {
    const double den = factorial(k) * factorial(j1 + j2 - j3 - k) * factorial(j1 - m1 - k) *
                       factorial(j2 + m2 - k) * factorial(j3 - j2 + m1 + k) * factorial(j3 - j1 - m2 + k);
    sum += ((k & 1) ? -1.0 : 1.0) / den;
  }
  const int ph = j1 - j2 - m3;
  return ((ph & 1) ? -1.0 : 1.0) * pref * sum;
}

using cplx = std::complex<double>;

// Real-basis vector m' of irrep l in terms of Condon-Shortley kets |l,m>:
//   m' > 0 : ((-1)^m' |m'> + |-m'>)/sqrt2     m' = 0 : |0>
//   m' < 0 : ((-1)^u |u> - |-u>)/(i sqrt2), u = -m'
// Returned as the (at most two) pairs (m, conj(coefficient)).
struct KetMix {
  int n;
  int m[2];
  cplx c[2];
};
KetMix real_vector_conj(int mp) {
  const double s = 1.0 / std::sqrt(2.0);
  KetMix k{};
  if (mp == 0) {
    k.n = 1;
    k.m[0] = 0;
    k.c[0] = 1.0;
    return k;
  }
  const int u = std::abs(mp);
  const double sg = (u & 1) ? -1.0 : 1.0;
  k.n = 2;
  k.m[0] = u;
  k.m[1] = -u;
  if (mp > 0) {
    k.c[0] = sg * s;
    k.c[1] = s;
  } else {
    // coefficients sg/(i sqrt2) = -i sg s and -1/(i sqrt2) = +i s; conjugated here
    k.c[0] = cplx(0.0, sg * s);
    k.c[1] = cplx(0.0, -s);
  }
  return k;
}

}  // namespace

std::vector<double> coupling_tensor(int l1, int l2, int l3) {
  const int n1 = 2 * l1 + 1, n2 = 2 * l2 + 1, n3 = 2 * l3 + 1;
  std::vector<double> out(static_cast<size_t>(n1) * n2 * n3, 0.0);
  if (l3 < std::abs(l1 - l2) || l3 > l1 + l2) return out;
  std::vector<cplx> t(out.size());
  for (int a = -l1; a <= l1; ++a) {
    const KetMix ka = real_vector_conj(a);
    for (int b = -l2; b <= l2; ++b) {
      const KetMix kb = real_vector_conj(b);
      for (int c = -l3; c <= l3; ++c) {
        const KetMix kc = real_vector_conj(c);
        cplx acc = 0.0;
        for (int i = 0; i < ka.n; ++i)
          for (int j = 0; j < kb.n; ++j)
            for (int k = 0; k < kc.n; ++k) {
              const double w = wigner_3j(l1, l2, l3, ka.m[i], kb.m[j], kc.m[k]);
              if (w != 0.0) acc += ka.c[i] * kb.c[j] * kc.c[k] * w;
            }
        t[(static_cast<size_t>(a + l1) * n2 + (b + l2)) * n3 + (c + l3)] = acc;
      }
    }
  }
  // The invariant is purely real for even l1+l2+l3 and purely imaginary otherwise.
  double re = 0.0, im = 0.0;
  for (const cplx& v : t) {
    re = std::max(re, std::abs(v.real()));
    im = std::max(im, std::abs(v.imag()));
  }
  double norm2 = 0.0;
  for (size_t i = 0; i < t.size(); ++i) {
    out[i] = (re >= im) ? t[i].real() : t[i].imag();
    norm2 += out[i] * out[i];
  }
  const double inv = 1.0 / std::sqrt(norm2);
  double sign = 0.0;
  for (double& v : out) {
    v *= inv;
    if (std::abs(v) < 1e-13) v = 0.0;
    if (sign == 0.0 && v != 0.0) sign = (v > 0.0) ? 1.0 : -1.0;
  }
  if (sign < 0.0)
    for (double& v : out) v = -v;
  return out;
}

bool build_path_table(int l_max, int nu_max, const std::vector<int>& out_l,
                      const std::vector<int>& out_parity, PathTable* table, const char** msg) {
  PathTable& T = *table;
  T = PathTable{};
  T.l_max = l_max;
  T.nu_max = nu_max;
  T.out_l = out_l;
  T.out_parity = out_parity;
  T.n_lm = (l_max + 1) * (l_max + 1);
  for (size_t o = 0; o < out_l.size(); ++o) {
    T.out_offset.push_back(T.n_LM);
    T.n_LM += 2 * out_l[o] + 1;
  }
  auto par = [](int lsum) { return (lsum & 1) ? -1 : 1; };
  std::vector<int> per_out(out_l.size(), 0);
  for (int nu = 1; nu <= nu_max; ++nu) {
    for (size_t o = 0; o < out_l.size(); ++o) {
      const int L = out_l[o], p = out_parity[o];
      std::vector<std::array<int, 4>> block;  // (l1, l2, L2, l3)
      if (nu == 1) {
        if (L <= l_max && par(L) == p) block.push_back({L, -1, -1, -1});
      } else if (nu == 2) {
        for (int l1 = 0; l1 <= l_max; ++l1)
          for (int l2 = 0; l2 <= l_max; ++l2)
            if (std::abs(l1 - l2) <= L && L <= l1 + l2 && par(l1 + l2) == p) block.push_back({l1, l2, -1, -1});
      } else {
        for (int l1 = 0; l1 <= l_max; ++l1)
          for (int l2 = 0; l2 <= l_max; ++l2)
            for (int L2 = std::abs(l1 - l2); L2 <= l1 + l2; ++L2)
              for (int l3 = 0; l3 <= l_max; ++l3)
                if (std::abs(L2 - l3) <= L && L <= L2 + l3 && par(l1 + l2 + l3) == p)
                  block.push_back({l1, l2, L2, l3});
      }
      std::sort(block.begin(), block.end());
      for (const auto& b : block) {
        T.paths.push_back(Path{nu, static_cast<int>(o), b[0], b[1], b[3], b[2]});
        ++per_out[o];
      }
    }
  }
  for (size_t o = 0; o < out_l.size(); ++o)
    if (per_out[o] == 0) {
      if (msg) *msg = "an output irrep cannot be reached by any coupling path";
      return false;
    }

  // sparse terms: chain the coupling tensors, merge slot permutations
  for (const Path& P : T.paths) {
    const int L = out_l[P.out];
    std::map<std::tuple<int, int, int, int>, double> acc;  // (M, i1, i2, i3) -> coef
    auto base = [](int l) { return l * l; };
    if (P.nu == 1) {
      for (int M = 0; M < 2 * L + 1; ++M) acc[{M, base(L) + M, -1, -1}] = 1.0;
    } else if (P.nu == 2) {
      const std::vector<double> C = coupling_tensor(P.l1, P.l2, L);
      const int n2 = 2 * P.l2 + 1, n3 = 2 * L + 1;
      for (int a = 0; a < 2 * P.l1 + 1; ++a)
        for (int b = 0; b < n2; ++b)
          for (int M = 0; M < n3; ++M) {
            const double v = C[(static_cast<size_t>(a) * n2 + b) * n3 + M];
            if (v == 0.0) continue;
            int i = base(P.l1) + a, j = base(P.l2) + b;
            if (i > j) std::swap(i, j);
            acc[{M, i, j, -1}] += v;
          }
    } else {
      const std::vector<double> C12 = coupling_tensor(P.l1, P.l2, P.L2);
      const std::vector<double> C23 = coupling_tensor(P.L2, P.l3, L);
      const int n2 = 2 * P.l2 + 1, nq = 2 * P.L2 + 1, n3 = 2 * P.l3 + 1, nM = 2 * L + 1;
      for (int a = 0; a < 2 * P.l1 + 1; ++a)
        for (int b = 0; b < n2; ++b)
          for (int c = 0; c < n3; ++c)
            for (int M = 0; M < nM; ++M) {
              double v = 0.0;
              for (int q = 0; q < nq; ++q)
                v += C12[(static_cast<size_t>(a) * n2 + b) * nq + q] * C23[(static_cast<size_t>(q) * n3 + c) * nM + M];
              if (v == 0.0) continue;
              std::array<int, 3> idx = {base(P.l1) + a, base(P.l2) + b, base(P.l3) + c};
              std::sort(idx.begin(), idx.end());
              acc[{M, idx[0], idx[1], idx[2]}] += v;
            }
    }
    std::vector<Term> terms;
    for (const auto& kv : acc) {
      if (std::abs(kv.second) < 1e-12) continue;
      // for nu = 1,2 the unused slots were stored as -1 in the LAST positions
      terms.push_back(Term{std::get<0>(kv.first), std::get<1>(kv.first), std::get<2>(kv.first),
                           std::get<3>(kv.first), kv.second});
    }
    T.terms.push_back(std::move(terms));
  }
  return true;
}

}  // namespace sc
