// Host-side coupling tables of the symmetric contraction (no HIP in this file).
//
// Wigner 3j symbols by the Racah sum, moved to the real spherical-harmonic basis,
// chained into the generalized coupling tensors of Algorithm 2 (arXiv 2504.10700,
// Section 4.1) and merged over slot permutations into sparse monomial terms.
#pragma once
#include <array>
#include <cstdint>
#include <vector>

namespace sc {

// Real-basis coupling tensor C(l1,l2,l3)[m1][m2][m3], row-major, unit Frobenius norm,
// first non-zero entry positive; all zero if the triangle rule fails.
std::vector<double> coupling_tensor(int l1, int l2, int l3);

struct Path {
  int nu, out, l1, l2, l3, L2;  // unused = -1
};

struct Term {      // coef * a[i1] * a[i2] * a[i3]  contributes to component M of its path
  int M;           // 0..2L
  int i1, i2, i3;  // component indices a = l*l+l+m, ascending; unused = -1
  double coef;
};

struct PathTable {
  int l_max = 0, nu_max = 0;
  std::vector<int> out_l, out_parity;
  std::vector<int> out_offset;          // first LM column of each output irrep
  int n_lm = 0, n_LM = 0;
  std::vector<Path> paths;              // global path order of the C ABI
  std::vector<std::vector<Term>> terms; // per path, sorted by (M, i1, i2, i3)
};

// Enumerates the paths and builds their sparse terms.  Returns false (with msg)
// if an output irrep has no path at all.
bool build_path_table(int l_max, int nu_max, const std::vector<int>& out_l,
                      const std::vector<int>& out_parity, PathTable* table, const char** msg);

}  // namespace sc
