// Host-side (fp64) closed-form fits of the DERF parameter families.
#pragma once
#include <vector>

namespace fs {

// a = v diag(w) v^T for symmetric a (n*n row-major, destroyed); w non-ascending; column j of v pairs with w[j].
void jacobi_eigh(int n, std::vector<double>& a, std::vector<double>& w, std::vector<double>& v);

// Writes one theta block (layout in favorsharp.h) from the statistics of one group.
// variant: fs_variant value.  Returns an fs_status value (0 ok, 1 bad variant, 3 singular statistics).
int fit_group(int variant, int d, const double* M1, const double* M2, const double* mu4, const double* mu5,
              double ridge, float* theta);

// Orthonormalises the rows of g (n x d, n <= d, row-major) in order (modified Gram-Schmidt, two passes) and scales
// row i to length len[i].  Returns false if a row has (numerically) no component outside the span of the earlier ones.
bool orthogonal_rows(int n, int d, const double* g, const double* len, double* out);

}  // namespace fs
