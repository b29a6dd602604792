"""Chunk-wise identities of the paper's Section 4.2.1, written out in fp64 numpy.

Test infrastructure only (same rules as gka_oracle.c).  These functions restate, for ONE chunk
of one (batch, head) pair, the formulas the paper gives for working with the chunk's initial
state H_0 instead of the per-token states H_1..H_C:

  zeta_c = prod_{i<=c} gamma_i,   M[j, c] = zeta_c / zeta_j  for c >= j, else 0
  H_c    = zeta_c H_0 + sum_j M[j, c] k_j k_j^T
  ||H_c||_F^2 = zeta_c^2 ||H_0||_F^2 + 2 zeta_c sum_j M[j, c] k_j^T H_0 k_j
                + column-sum(((G o G) M) o M)_c,            G = K K^T (Gram matrix of the keys)
  H_c xi = zeta_c H_0 xi + sum_{j<=c} M[j, c] k_j (k_j^T xi)

The mask is built in log space, M[j, c] = exp(G_c - G_j) (Appendix B.2, "Derivatives for
Gating").  The tests compare each of these against the step-by-step recurrence of the C oracle.
"""
import numpy as np


def decay_mask(gamma):
    """gamma: [C] gates of one chunk -> (zeta [C], M [C, C]) with M[j, c] = zeta_c / zeta_j, c >= j."""
    g = np.log(np.asarray(gamma, dtype=np.float64))
    G = np.cumsum(g)
    zeta = np.exp(G)
    C = G.shape[0]
    M = np.zeros((C, C), dtype=np.float64)
    for j in range(C):
        for c in range(j, C):
            M[j, c] = np.exp(G[c] - G[j])
    return zeta, M


def unrolled_states(H0, K, gamma):
    """All per-token states of a chunk from its initial state. K: [C, d] rows k_j. -> [C, d, d]."""
    zeta, M = decay_mask(gamma)
    C, d = K.shape
    out = np.empty((C, d, d), dtype=np.float64)
    for c in range(C):
        Hc = zeta[c] * H0
        for j in range(C):
            Hc = Hc + M[j, c] * np.outer(K[j], K[j])
        out[c] = Hc
    return out


def frobenius_norms(H0, K, gamma):
    """||H_1||_F .. ||H_C||_F by the three-term expansion with the column-sum formula."""
    zeta, M = decay_mask(gamma)
    term1 = zeta ** 2 * np.sum(H0 * H0)
    quad = np.einsum("jd,de,je->j", K, H0, K)            # k_j^T H_0 k_j
    term2 = 2.0 * zeta * np.sum(quad[:, None] * M, axis=0)
    G = K @ K.T
    term3 = np.sum(((G * G) @ M) * M, axis=0)
    return np.sqrt(term1 + term2 + term3)


def chunk_matvec(H0, K, gamma, Xi):
    """Row c of the result is H_c xi_c for the rows xi_c of Xi [C, d], without forming H_c."""
    zeta, M = decay_mask(gamma)
    P = Xi @ K.T                      # P[c, j] = k_j^T xi_c
    return zeta[:, None] * (Xi @ H0.T) + (P * M.T) @ K


def chunk_end_state(S0, A, Kmat, gamma):
    """State after the chunk: zeta_C S_0 + sum_j M[j, C] a_j k_j^T (A = K for H, A = V for U)."""
    zeta, M = decay_mask(gamma)
    return zeta[-1] * S0 + (A * M[:, -1][:, None]).T @ Kmat
