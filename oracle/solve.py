"""Oracle for the optimal decomposition (Section 3.2, Eq. 11 and Eq. 12) -- TEST
INFRASTRUCTURE.  Plain exhaustive search over the naturals, as the paper says."""
from __future__ import annotations


def normalisation_blocks(B_A, B_S, B_D, B_GPU, alpha_A=1.0, alpha_S=1.0, alpha_D=1.0, limit=10**6):
    """Smallest a with (alpha_A B_A + alpha_S B_S)/a + alpha_D B_D <= B_GPU, or None."""
    for a in range(1, limit + 1):
        if (alpha_A * B_A + alpha_S * B_S) / a + alpha_D * B_D <= B_GPU:
            return a
    return None


def aggregation_blocks(B_S, B_X, B_GPU, beta_S=1.0, beta_X=1.0, max_c=64, max_b=4096):
    """(b, c) minimising b*c subject to beta_S B_S/b + beta_X B_X/c <= B_GPU; among
    equal products the smaller c.  None if nothing in the searched box fits."""
    best = None
    for c in range(1, max_c + 1):
        for b in range(1, max_b + 1):
            if beta_S * B_S / b + beta_X * B_X / c <= B_GPU:
                if best is None or b * c < best[0] * best[1]:
                    best = (b, c)
                break
    return best
