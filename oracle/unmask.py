"""Oracle: confidence-aware unmasking of the active block.

Steps, in the paper's order and notation:
  * Eq. 4 (section 3.1): for every masked position i of the active block,
    c_i = max softmax(z_i), xhat_i = argmax softmax(z_i)  (lowest id on ties);
  * Eq. 10 (section 3.3): tau = tau0 * (1 - alpha * (1 - r_mask)), r_mask taken from
    the state before this step's commit; r_mask = (m + extra_masked) / (K + extra_total)
    where m is the number of masked positions of the block (extra_* = 0 gives the
    block-only reading, extra_* = s the whole-query reading);
  * Eq. 9 + the sentence before it: commit every masked i with c_i >= tau; when no
    masked position reaches tau, commit the single masked position of highest
    confidence (lowest position on ties);
  * Eq. 5: committed positions take xhat_i and are never re-masked, all other
    positions are unchanged;
  * block termination (end of section 3.1): block_done <=> no masked position left;
  * early exit (section 3.3): eos_seen becomes (and stays) 1 when a token committed
    in this call equals eos_id with confidence >= tau_eos.
Float64 throughout.  Test infrastructure only -- never imported by the product path.
"""
from __future__ import annotations

import numpy as np


def row_confidence(z):
    """Eq. 4 for one row of logits z (float64): returns (c, xhat, gap).

    c = max_j softmax(z)_j = 1 / sum_j exp(z_j - z_max); xhat = lowest index attaining
    the maximum; gap = difference between the two largest softmax probabilities.
    """
    z = np.asarray(z, dtype=np.float64)
    xhat = int(np.argmax(z))            # numpy returns the first maximal index
    e = np.exp(z - z[xhat])
    denom = e.sum()
    c = 1.0 / denom
    if z.shape[0] > 1:
        e[xhat] = -1.0
        second = e.max() / denom
    else:
        second = 0.0
    return c, xhat, c - second


def dynamic_threshold(tau0, alpha, m, K, extra_masked=0, extra_total=0):
    """Eq. 10."""
    r_mask = (m + extra_masked) / float(K + extra_total)
    return tau0 * (1.0 - alpha * (1.0 - r_mask))


def confidence_unmask(logits, tokens, masked, tau0, alpha, eos_id=-1, tau_eos=None,
                      extra_masked=0, extra_total=0, eos_seen=None, V=None):
    """logits float64 [B,K,ld] (first V entries of a row are valid); tokens int [B,K];
    masked uint8 [B,K].  Returns a dict with the updated state and diagnostics:
      tokens, masked, n_committed[B], block_done[B], eos_seen[B],
      confidence[B,K] (nan where not masked), xhat[B,K] (-1 where not masked),
      gap[B,K] (top-2 probability gap, nan where not masked), tau[B], fallback[B].
    """
    logits = np.asarray(logits)
    B, K = tokens.shape
    if V is None:
        V = logits.shape[2]
    if tau_eos is None:
        tau_eos = tau0
    tokens = np.array(tokens, dtype=np.int64, copy=True)
    masked_in = np.asarray(masked)
    masked_out = np.array(masked, dtype=np.uint8, copy=True)
    eos_out = np.zeros(B, dtype=np.uint8) if eos_seen is None else np.array(eos_seen, dtype=np.uint8, copy=True)
    n_committed = np.zeros(B, dtype=np.int64)
    block_done = np.zeros(B, dtype=np.uint8)
    conf = np.full((B, K), np.nan)
    gap = np.full((B, K), np.nan)
    xhat = np.full((B, K), -1, dtype=np.int64)
    tau = np.full(B, np.nan)
    fallback = np.zeros(B, dtype=np.uint8)
    for b in range(B):
        M = [i for i in range(K) if masked_in[b, i] != 0]
        m = len(M)
        if m == 0:
            block_done[b] = 1
            continue
        for i in M:
            c, xh, gp = row_confidence(np.asarray(logits[b, i, :V], dtype=np.float64))
            conf[b, i], xhat[b, i], gap[b, i] = c, xh, gp
        tau[b] = dynamic_threshold(tau0, alpha, m, K, extra_masked, extra_total)
        C = [i for i in M if conf[b, i] >= tau[b]]
        if not C:
            best = M[0]
            for i in M[1:]:
                if conf[b, i] > conf[b, best]:
                    best = i
            C = [best]
            fallback[b] = 1
        for i in C:
            tokens[b, i] = xhat[b, i]
            masked_out[b, i] = 0
            if eos_id >= 0 and xhat[b, i] == eos_id and conf[b, i] >= tau_eos:
                eos_out[b] = 1
        n_committed[b] = len(C)
        block_done[b] = 1 if (m - len(C)) == 0 else 0
    return {
        "tokens": tokens, "masked": masked_out, "n_committed": n_committed, "block_done": block_done,
        "eos_seen": eos_out, "confidence": conf, "xhat": xhat, "gap": gap, "tau": tau, "fallback": fallback,
    }
