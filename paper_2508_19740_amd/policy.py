"""Caller-side policy that is not part of the kernels' path: how many tokens to keep."""
import math


def token_budget(n_tokens: int, pruning_rate: float, minimum: int = 20) -> int:
    """k for a context of n_tokens (paper appendix, language-modeling details): the kept share of
    the sequence rounded down, but at least `minimum` tokens; 98 % pruning gives 81 of 4096 and
    163 of 8192."""
    kept = int(math.floor(n_tokens * (1.0 - pruning_rate) + 1e-9))
    return max(minimum, kept)
