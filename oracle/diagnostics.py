"""Per-position statistics of a decode iteration (oracle side; test infrastructure only).

The quantities the paper's analysis is written in (Sec. 3 "Motivation and
Analysis", Eq. beta = 1 - D_TV; Prop. "SJD Collision Probability"; the Hamming
distance between consecutive drafts of Sec. 3 and Sec. 5.3), each as its
definition, in fp64:

  acceptance rate       beta = 1 - D_TV(p, q),  D_TV = 1/2 sum_v |p_v - q_v|
  collision probability C(p, q) = sum_v p_v q_v     (independent draws X ~ p, Y ~ q)
  Renyi-2 entropy       H_2(p) = -log sum_v p_v^2
  entropy bound         C(p, q) <= exp(-(H_2(p) + H_2(q)) / 2)
  Hamming distance      number of window positions whose draft token changed
"""
import numpy as np


def total_variation(p, q):
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    return 0.5 * np.abs(p - q).sum()


def acceptance_rate(p, q):
    """beta = 1 - D_TV(p, q): the probability that MRS(p, q, X ~ q) accepts."""
    return 1.0 - total_variation(p, q)


def collision_probability(p, q):
    """Pr[X = Y] for independent X ~ p, Y ~ q."""
    return float(np.dot(np.asarray(p, dtype=np.float64), np.asarray(q, dtype=np.float64)))


def renyi2_entropy(p):
    p = np.asarray(p, dtype=np.float64)
    return -np.log(np.dot(p, p))


def collision_bound(p, q):
    """exp(-(H_2(p) + H_2(q)) / 2), the upper bound of the collision probability."""
    return float(np.exp(-0.5 * (renyi2_entropy(p) + renyi2_entropy(q))))


def row_statistics(p, q):
    """The four numbers kept per window position: (beta, C, sum p^2, sum q^2);
    the entropy bound is sqrt of the product of the last two."""
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    return (acceptance_rate(p, q), collision_probability(p, q), float(np.dot(p, p)), float(np.dot(q, q)))


def hamming(x_old, x_new):
    """Number of positions at which two drafts of the same positions differ."""
    x_old = np.asarray(x_old)
    x_new = np.asarray(x_new)
    assert x_old.shape == x_new.shape
    return int((x_old != x_new).sum())
