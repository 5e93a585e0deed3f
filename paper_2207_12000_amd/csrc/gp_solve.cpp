// Optimal graph decomposition (Section 3.2, Eq. 11 and Eq. 12): the smallest
// block counts whose working set fits the GPU volume.
#include <cmath>

#include "gp_internal.h"

using namespace gp;

extern "C" gp_status gp_solve_normalisation_blocks(double B_A, double B_S, double B_D, double B_GPU, double alpha_A,
                                                   double alpha_S, double alpha_D, int64_t* a)
{
    if (!a) return fail(GP_ERR_INVALID_ARG, "output pointer is NULL");
    *a = 0;
    if (!(B_A >= 0) || !(B_S >= 0) || !(B_D >= 0) || !(B_GPU > 0) || !(alpha_A >= 0) || !(alpha_S >= 0) || !(alpha_D >= 0))
        return fail(GP_ERR_INVALID_ARG, "volumes must be >= 0 (B_GPU > 0) and coefficients >= 0");
    const double fixed = alpha_D * B_D, split = alpha_A * B_A + alpha_S * B_S;
    if (fixed > B_GPU || (fixed == B_GPU && split > 0))
        return fail(GP_ERR_UNSUPPORTED, "the degree matrix term alone (%g) does not leave room in %g", fixed, B_GPU);
    if (split == 0) {
        *a = 1;
        return GP_OK;
    }
    // one free parameter: start from the real-valued bound and settle on the exact natural
    double guess = std::ceil(split / (B_GPU - fixed));
    if (!(guess >= 1)) guess = 1;
    if (guess > 9.0e18) return fail(GP_ERR_OVERFLOW, "block count does not fit int64");
    int64_t k = (int64_t)guess;
    while (k > 1 && split / (double)(k - 1) + fixed <= B_GPU) --k;
    while (split / (double)k + fixed > B_GPU) ++k;
    *a = k;
    return GP_OK;
}

extern "C" gp_status gp_solve_aggregation_blocks(double B_S, double B_X, double B_GPU, double beta_S, double beta_X,
                                                 int64_t max_c, int64_t* b, int64_t* c)
{
    if (!b || !c) return fail(GP_ERR_INVALID_ARG, "output pointer is NULL");
    *b = *c = 0;
    if (!(B_S >= 0) || !(B_X >= 0) || !(B_GPU > 0) || !(beta_S >= 0) || !(beta_X >= 0) || max_c < 1)
        return fail(GP_ERR_INVALID_ARG, "volumes must be >= 0 (B_GPU > 0), coefficients >= 0, max_c >= 1");
    const double s = beta_S * B_S, x = beta_X * B_X;
    // exhaustive over c; for each c the smallest feasible b is fixed by the constraint
    int64_t best_b = 0, best_c = 0;
    double best_prod = 0;
    for (int64_t cc = 1; cc <= max_c; ++cc) {
        const double room = B_GPU - x / (double)cc;
        if (room < 0 || (room == 0 && s > 0)) continue;
        int64_t bb = 1;
        if (s > 0) {
            double g = std::ceil(s / room);
            if (!(g >= 1)) g = 1;
            if (g > 4.0e18) continue;
            bb = (int64_t)g;
            while (bb > 1 && s / (double)(bb - 1) + x / (double)cc <= B_GPU) --bb;
            while (s / (double)bb + x / (double)cc > B_GPU) ++bb;
        }
        const double prod = (double)bb * (double)cc;
        if (best_c == 0 || prod < best_prod) {
            best_prod = prod;
            best_b = bb;
            best_c = cc;
        }
        // a larger c can only win with a smaller b; once b is 1 nothing better follows
        if (bb == 1) break;
        if ((double)cc >= best_prod) break;  // every later pair has a product above the best
    }
    if (best_c == 0) return fail(GP_ERR_UNSUPPORTED, "no (b, c) with c <= %lld fits %g", (long long)max_c, B_GPU);
    *b = best_b;
    *c = best_c;
    return GP_OK;
}
