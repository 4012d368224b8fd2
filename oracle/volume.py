"""Eq. 2 of the paper, written out (test infrastructure): the ratio gamma of the total network data
volume of standard training to that of lazy message passing.

    gamma = ( 1 + B (2 sum_H / M + H0 / (M R)) ) / ( 1 + sum_C / M + B (sum_H / (M R) + H0 / (M R)) )

B boundary nodes per worker, R training rounds, H0 feature size, sum_H the intermediate representation
sizes H_1 .. H_{K-1} added up, sum_C the added classifier sizes, M the model size.
"""


def gamma(B: float, R: float, H0: float, sum_H: float, sum_C: float, M: float) -> float:
    num = 1.0 + B * (2.0 * sum_H / M + H0 / (M * R))
    den = 1.0 + sum_C / M + B * (sum_H / (M * R) + H0 / (M * R))
    return num / den
