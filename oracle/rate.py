"""Function transfer rate control of Sec. 6.1, and the step from rates to the
integer weights the chunk interleave takes.

Sec. 6.1: the least rate a function needs is its data size over the time its
SLO leaves for the transfer, Rate_least = data_size / (L_slo - L_infer). What
the link has beyond the sum of all least rates, Rate_idle = BW_all - sum of
Rate_least, goes to the function with the tightest SLO.

Readings where the text is silent:
  * tightest SLO = smallest L_slo - L_infer (the time left for the transfer);
    ties go to the lowest function index;
  * a function whose SLO leaves no time (L_slo <= L_infer) is an input error;
  * when the least rates already exceed the link (Rate_idle <= 0) nothing is
    added: the functions share in proportion to their least rates;
  * weights: the share of the weight total, `total` = 64 by default, that
    equals the function's share of the rate sum, rounded half up, at least 1.
    (One unit is then 1/64 of the link.) All arithmetic is IEEE double in the
    order written here. The rule itself fixes the weights only up to the rounding
    of a quotient that may fall within an ulp of a half: an implementation that
    evaluates the expression in another order is still correct if every weight
    differs from these by at most one unit. The library's host code happens to
    use the same order, so its tests can ask for equality; that is a property of
    the two implementations as they stand, not of the rule (the pins of this
    module - hand values, unit invariance - hold for either order).

TEST INFRASTRUCTURE ONLY (see the package docstring).
"""
import math

from . import OracleError, EINVAL


def least_rates(data_size, l_slo, l_infer):
    rates = []
    for size, slo, infer in zip(data_size, l_slo, l_infer):
        slack = float(slo) - float(infer)
        if not (slack > 0.0) or size < 0:
            raise OracleError(EINVAL, "the SLO leaves no time for the transfer")
        rates.append(float(size) / slack)
    return rates


def allocate_rates(data_size, l_slo, l_infer, bw_all):
    """Rate of every function: its least rate, plus the idle rate for the tightest one."""
    if len(data_size) == 0 or not (float(bw_all) > 0.0):
        raise OracleError(EINVAL, "no functions or no bandwidth")
    rates = least_rates(data_size, l_slo, l_infer)
    total = 0.0
    for r in rates:
        total = total + r
    idle = float(bw_all) - total
    if idle > 0.0:
        tight = 0
        for i in range(1, len(rates)):
            if float(l_slo[i]) - float(l_infer[i]) < float(l_slo[tight]) - float(l_infer[tight]):
                tight = i
        rates[tight] = rates[tight] + idle
    return rates


def rates_to_weights(rates, total=64):
    s = 0.0
    for r in rates:
        s = s + r
    if not (s > 0.0):
        return [1] * len(rates)
    out = []
    for r in rates:
        w = int(math.floor(r / s * float(total) + 0.5))
        out.append(w if w >= 1 else 1)
    return out


def slo_weights(data_size, l_slo, l_infer, bw_all, total=64):
    return rates_to_weights(allocate_rates(data_size, l_slo, l_infer, bw_all), total)
