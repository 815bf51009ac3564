"""Oracle: attenuation-guided suffix selection (paper Eq. 7, Fig. 4).

With the prompt of length p_L, blocks I_n = {p_L + nK, ..., p_L + (n+1)K - 1} and current block c,
the kept index set is the blocks up to c + w together with the final position of the sequence;
restricted to the suffix (the positions after block c) that is the w blocks nearest to the current
one plus the trailing position.  Written with absolute positions, as in the paper, then made
relative to the start of the suffix.  Reading taken where the paper's text is loose: the final
position is the last generated position p_L + L - 1 (the printed index p_L + L is one past the end
for 0-based positions), and a window that reaches the end of the sequence simply stops there.
Test infrastructure only -- never imported by the product path.
"""
from __future__ import annotations


def suffix_keep_indices(p_L: int, L: int, K: int, c: int, w: int, keep_trailing: bool = True):
    """Returns the kept suffix positions relative to the start of the suffix (sorted list)."""
    N = L // K
    assert L == N * K and 0 <= c < N
    suffix_start = p_L + (c + 1) * K
    kept = set()
    for n in range(c + 1, min(c + w, N - 1) + 1):          # blocks c+1 .. c+w that exist
        for pos in range(p_L + n * K, p_L + (n + 1) * K):
            kept.add(pos)
    last = p_L + L - 1
    if keep_trailing and last >= suffix_start:
        kept.add(last)
    return sorted(pos - suffix_start for pos in kept)
