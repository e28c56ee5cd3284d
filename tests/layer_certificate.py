"""Layer-by-layer certificate for a network whose hidden activations are rounded to bf16 (test code).

End to end, two correct evaluations of a deep bf16 network disagree: an activation whose exact value lies next
to a rounding boundary rounds one way with fp32 sums and the other way with fp64 sums, and every such one-step
difference perturbs the next layer.  Layer by layer nothing compounds: feed the activations ONE side produced
for layer l to the other side's layer l + 1 and compare the outputs.  What remains is the error of the fp32
accumulation alone, and a rounded output can only differ where the exact pre-activation lies within that error
of a rounding boundary -- and then only by landing on the neighbouring bf16 value.

Bound on the accumulation error of one output, sum_i a_i w_i + b over K terms: the products of two bf16 numbers
are exact in fp32, every addition rounds with unit roundoff u = 2^-24, so the error is at most
(number of additions) * u * sum_i |a_i w_i| in the worst case and about sqrt(number of additions) * u * (typical
partial sum) when the rounding errors are independent.  The certificate uses

    err = ERR_FACTOR * u * sum_i |a_i w_i|        (per output element, computed by the oracle in fp64)

with ERR_FACTOR = 8: sum |a_i w_i| is itself ~sqrt(K) times the typical partial sum for weights of random sign,
so this is the probabilistic bound with a safety factor of 8, and a small fraction of the worst-case bound K * u
* sum |a_i w_i| (K = 1664 for the 5 x 5 convolutions).  It keeps the band around a bf16 rounding boundary
(relative width 2^-8) in which either neighbour is accepted to a few per cent of all activations.
"""
import numpy as np

from oracle import made_oracle as O

U32 = 2.0 ** -24
ERR_FACTOR = 8.0


def sum_error(abs_product_sum):
    """err per output element from sum_i |a_i w_i| (+ |b|)."""
    return ERR_FACTOR * U32 * np.asarray(abs_product_sum, dtype=np.float64)


def certify_rounded(pre, err, got):
    """pre: exact pre-activation (bias included, before ReLU), fp64.  got: the other side's activation after ReLU
    and bf16 rounding (as float).  Returns (ok, exact, near):
      ok    -- got lies between bf16(relu(pre - err)) and bf16(relu(pre + err)) (rounding is monotone, so this is
               exactly "got is the rounding of SOME value within err of pre")
      exact -- got == bf16(relu(pre))
      near  -- the two ends of that interval differ (pre is within err of a rounding boundary, or of 0)."""
    lo = O.round_to_bf16(np.maximum(pre - err, 0.0))
    hi = O.round_to_bf16(np.maximum(pre + err, 0.0))
    mid = O.round_to_bf16(np.maximum(pre, 0.0))
    got = np.asarray(got, dtype=np.float64)
    return (got >= lo) & (got <= hi), got == mid, lo != hi


def certify_plain(pre, err, got):
    """Outputs that are not rounded (fp32 activations, logits): |got - pre| <= err + one fp32 ulp of pre."""
    got = np.asarray(got, dtype=np.float64)
    return np.abs(got - pre) <= err + np.abs(pre) * 2.0 ** -23


def summarize(name, ok, exact, near):
    return (f"{name}: {int((~ok).sum())} of {ok.size} outside the certificate, {float(exact.mean()) * 100:.3f} % "
            f"bit-identical, {float(near.mean()) * 100:.3f} % within the error of a rounding boundary")
