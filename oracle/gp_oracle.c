/* Oracle for the K-hop feature precompute -- TEST INFRASTRUCTURE, not product code.
 *
 * One hop of X_k = A^ X_{k-1} written out as the plain definition: a loop over
 * the adjacency list (COO), in fp64, one fused scale-and-add per non-zero and
 * column.  The three operators:
 *   sym  : A^ = D~^-1/2 A~ D~^-1/2            (Eq. 1; the filter of Algorithm 1)
 *   mean : A^ = D^-1 A                          (row-normalised mean)
 *   sum  : A^ = A (with whatever diagonal the non-zero list holds)
 * deg[] is the row sum of the 0/1 matrix whose non-zeros are listed.  A weight
 * that needs a zero degree is 0.  The paper's blocks (Section 3.2) change the
 * schedule of this sum, not its value, so the oracle has no blocks at all.
 *
 * Entries [e_lo, e_hi) are processed in list order and added into Y, which the
 * caller has zeroed: calling it on disjoint ranges that do not share a row is
 * the same computation (each row still sees its entries in list order).
 *
 * Build: gcc -O2 -shared -fPIC (no fast-math, no reassociation).
 */
#include <math.h>
#include <stdint.h>

enum { GPO_SYM = 0, GPO_MEAN = 1, GPO_SUM = 2 };

static double edge_weight(int agg, int32_t deg_row, int32_t deg_col)
{
    switch (agg) {
    case GPO_SYM:
        if (deg_row <= 0 || deg_col <= 0) return 0.0;
        return 1.0 / sqrt((double)deg_row * (double)deg_col);
    case GPO_MEAN:
        if (deg_row <= 0) return 0.0;
        return 1.0 / (double)deg_row;
    default:
        return 1.0;
    }
}

/* Y[row[e], :] += w_e * X[col[e], :]  for e in [e_lo, e_hi).
 * X and Y are row-major n x d doubles with no padding.  Returns 0, or -1 on a
 * bad argument (nothing written). */
int gpo_hop_range(int64_t e_lo, int64_t e_hi, const int32_t *row, const int32_t *col,
                  const int32_t *deg, int agg, int64_t d, const double *X, double *Y)
{
    if (e_lo < 0 || e_hi < e_lo || d <= 0 || agg < 0 || agg > 2) return -1;
    for (int64_t e = e_lo; e < e_hi; ++e) {
        const int64_t i = row[e], j = col[e];
        const double w = edge_weight(agg, deg[i], deg[j]);
        const double *x = X + j * d;
        double *y = Y + i * d;
        for (int64_t c = 0; c < d; ++c) y[c] += w * x[c];
    }
    return 0;
}
