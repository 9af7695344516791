"""Oracle outputs for a sample of tokens of a layer too large to run whole on the CPU (indexing only)."""
import numpy as np


def oracle_out_for_tokens(O, x: np.ndarray, weights: dict, plan: dict, tokens, *, act: str, residual=None) -> np.ndarray:
    """out[t] for the listed tokens from the oracle's own functions, with the sampled rows of one expert going
    through that expert's FFN together (``O.sampled_tokens_forward`` converts an expert's matrices to float64
    once per token and choice: minutes for a few hundred tokens of the large workload).  Only indexing happens
    here: the kept choices (t, j) of the sampled tokens become the rows of a reduced dispatched batch, ordered
    by expert; ``O.expert_ffn`` computes that batch and ``O.combine`` the weighted sum.  ``plan`` carries the
    oracle's routing of the whole batch (topk_idx, topk_w, assign_to_row).  Checked against
    ``O.layer_forward`` in tests/test_oracle_pins.py."""
    toks = np.asarray(tokens, dtype=np.int64)
    T, k = plan["topk_idx"].shape
    n = len(toks)
    E = int(weights["w_router"].shape[1])
    pairs = [(int(plan["topk_idx"][t, j]), j, i) for i, t in enumerate(toks) for j in range(k)
             if plan["assign_to_row"][j * T + t] >= 0]
    pairs.sort()                                              # by expert, then choice, then sample position
    a2r = np.full(k * n, -1, dtype=np.int64)
    offsets = np.zeros(E + 1, dtype=np.int64)
    rows = np.zeros((len(pairs), x.shape[1]), dtype=np.float64)
    for r, (e, j, i) in enumerate(pairs):
        a2r[j * n + i] = r
        offsets[e + 1] += 1
        rows[r] = x[toks[i]]
    offsets = np.cumsum(offsets)
    yd = O.expert_ffn(rows, offsets, weights, act)
    res = None if residual is None else np.asarray(residual)[toks]
    return O.combine(yd, a2r, np.asarray(plan["topk_w"])[toks], res)
