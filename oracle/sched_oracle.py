"""Oracle of the proxy's scheduling arithmetic -- TEST INFRASTRUCTURE ONLY.

Plain Python, written from the paper: the offloading-ratio bounds of Sec. 3.4.1 (Eq. 1, 2, 3),
the load-aware offloading decision of Sec. 3.4.3 (Algorithm 1) in the listing's order and
notation, and the choice of a recorded graph of Sec. 3.2.2.  Exact rational arithmetic
(`fractions.Fraction`) wherever a comparison decides, so the oracle's decision does not depend on
floating-point rounding.  It shares nothing with the library and never imports it.

Readings: the comparisons of C1 and C2 are strict, as printed; `attn_max_tokens` is computed by
the listing and used by neither condition; a request's `max_token` is its prompt plus the most it
may generate and `used_token` the tokens it holds now.
"""
from fractions import Fraction


def offload_bound_mem(hbm_p, bw_p, hbm_d, bw_d):
    """Eq. 1: min(sum HBM_pi / HBM_d, sum BW_pi / BW_d)."""
    return min(Fraction(sum(Fraction(x) for x in hbm_p)) / Fraction(hbm_d),
               Fraction(sum(Fraction(x) for x in bw_p)) / Fraction(bw_d))


def offload_bound_comp(b_max, b_tpot):
    """Eq. 2: (B_max - B_TPOT) / B_TPOT."""
    return (Fraction(b_max) - Fraction(b_tpot)) / Fraction(b_tpot)


def offload_bound(ob_mem, ob_comp):
    """Eq. 3."""
    return min(ob_mem, ob_comp)


def need_offload(req, LR, OR, OB):
    """Algorithm 1.  req = (max_token, used_token); LR, OR lists of such pairs; OB the bound."""
    OB = Fraction(OB)
    need = 0
    attn_max_tokens = sum(r[0] for r in OR)          # computed by the listing, not used below
    attn_used_tokens = sum(r[1] for r in OR)
    decode_used_tokens = sum(r[1] for r in LR)
    if attn_used_tokens + req[0] < decode_used_tokens * OB:                       # C1
        need = 1
    elif attn_used_tokens + req[1] < decode_used_tokens * OB and len(OR) + 1 < len(LR) * OB:   # C2
        need = 1
    del attn_max_tokens
    return need


def graph_capacity(n, interval, max_capacity):
    """Smallest recorded capacity (multiples of `interval`, at least one) holding n rows, or -1."""
    if n < 0 or interval <= 0 or max_capacity < interval:
        return -1
    c = interval
    while c < n:
        c += interval
    return c if c <= max_capacity else -1
