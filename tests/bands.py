"""Error bounds that the tests derive from the arithmetic instead of choosing a tolerance.  Plain numpy; no code of
the method.

Ranking key of a list build (Algorithm 1 line 3): per head (z - m) - log S with z the scaled logit, m the maximum
and S the sum of exp(z_i - m) over the s keys; the key of a KV head is the maximum over its group.

Logits.  A logit is a sum of n = 128 products.  Accumulated in fp32 in any order, |fl(sum) - sum| <= (n - 1) u
sum|c_i k_i| <= (n - 1) u |c| |k| to first order (Cauchy-Schwarz); ACC_TERMS = 129 also covers a rounded product
(fp32 inputs) and the multiplication by the scale: eps_z = ACC_TERMS u |c| max|k| scale.  z and m then move by at
most eps_z each, every term of S by a factor within e^(+-2 eps_z), so log S by at most 2 eps_z, and a maximum over
heads by no more than its largest argument does: 4 eps_z.  On inputs whose dot products are exact in fp32 (small
integers times powers of two) every route computes the same z and m, and this part is zero.

Denominators.  The fixed-order route sums floor(exp(x) 2^40) as integers, exp by a polynomial within 2^-22
relative: S is short by at most s 2^-40 (S >= 1) and off by 2^-22 relative.  The matrix-core route keeps a running
fp32 sum: hardware exponential within 2^-22 relative of exp of its fp32 argument, the argument scaled to base two
in fp32 (terms that matter have |x| < 32: another 32 * 2^-24), one addition and at most one rescaling (a product
with a hardware exponential) per step of 32 keys, a tree over a step's terms and the merges of lane halves and
blocks: at most s / 32 + 64 operations deep, each within 2 u (u = 2^-24) relative.  log itself: 2^-22 absolute.

KEY_ROUND covers the roundings of the key itself (three operations on magnitudes below 64).  The matrix-core route
forms a key as fma(acc, scale, -(m + log S)): the offset is rounded once at magnitude up to |c| max|k| scale, hence
another 2^-23 |c| max|k| scale there, and as much again because the maximum is kept in base two and converted
back, also on inputs whose dot products are exact."""
import numpy as np

ACC_TERMS = 129
KEY_ROUND = 3 * 2.0 ** -18
U_NEAREST = 2.0 ** -24     # fp32 round to nearest: the fixed-order route on either side
U_TRUNCATE = 2.0 ** -23    # an accumulation that may truncate: what is assumed of the matrix cores


def _norms(Qc_group, K_kv):
    c = np.sqrt((np.asarray(Qc_group, np.float64) ** 2).sum(-1)).max()
    k = np.sqrt((np.asarray(K_kv, np.float64) ** 2).sum(-1)).max()
    return c, k


def denominator_bound(s, running_fp32):
    """|computed log S - exact log S| given exact exponents, for s keys."""
    if running_fp32:
        return 2.0 ** -22 + 32 * 2.0 ** -24 + 2 * (s / 32 + 64) * U_NEAREST + 2.0 ** -22
    return s * 2.0 ** -40 + 2.0 ** -22 + 2.0 ** -22


def key_error_bound(Qc_group, K_kv, scale, u, running_fp32=False, exact_dots=False):
    """|computed key - exact key| for one route: logits accumulated with unit roundoff u, denominators summed as
    2^-40 fixed point (running_fp32=False) or as a running fp32 sum.  Qc_group [G][d], K_kv [s][d]."""
    c, k = _norms(Qc_group, K_kv)
    eps_z = 0.0 if exact_dots else ACC_TERMS * u * c * k * float(scale)
    offset = 2.0 ** -22 * c * k * float(scale) if running_fp32 else 0.0
    return 4 * eps_z + offset + denominator_bound(len(K_kv), running_fp32) + KEY_ROUND


def key_band(Qc_group, K_kv, scale, exact_dots=False):
    """How far from the rho-th key an id may lie when the matrix-core route and the fixed-order route disagree on
    its membership.  With E the sum of the two routes' error bounds: an id a that only the first lists and an id b
    that only the second lists satisfy key(b) >= rho-th >= key(a) on the second route and key'(a) >= key'(b) on the
    first, so key(a) >= key'(a) - E >= key'(b) - E >= key(b) - 2E: both lie within 2E of the rho-th key."""
    return 2 * (key_error_bound(Qc_group, K_kv, scale, U_NEAREST, False, exact_dots) +
                key_error_bound(Qc_group, K_kv, scale, U_TRUNCATE, True, exact_dots))
