"""Plain numpy/float64 oracle of the whole drafter with tree drafting (test infrastructure only).

Embedding -> blocks -> final RMSNorm -> LM head for the prefix (Sec. 3.1 of the paper), then a
tree (N_1..N_gamma) drafted as batch generation (Sec. 4.1): the N_i children of a branch are its N_i
most probable tokens, child j of branch b is row b * N_i + j and continues from b's states.
Activations between stages are rounded to bf16 like the stored tensors they stand for.
"""
import numpy as np

import oracle


def _rb(a):
    return oracle._round_bf16(a)


def prefill(w, tokens, eps=1e-5):
    """w: embedding (V,dm), blocks (list of weight dicts for oracle.block_fwd), norm_f (dm), lm_head (V,dm).
    Returns logits (1,V), conv states (nl,1,D,K-1), ssm states (nl,1,D,N)."""
    hid = oracle.embedding(tokens, w["embedding"])[None]
    convs, ssms = [], []
    for bw in w["blocks"]:
        hid, cs, hs = oracle.block_fwd(bw, hid, eps=eps)
        hid = _rb(hid)
        convs.append(cs)
        ssms.append(hs)
    last = _rb(oracle.rmsnorm(hid[0, -1:], w["norm_f"], eps))
    return _rb(oracle.linear(last, w["lm_head"])), np.stack(convs), np.stack(ssms)


def draft(w, tree, logits, conv, ssm, eps=1e-5):
    """Returns per position the draft tokens, plus the per-position logits and the smallest gap
    between the last chosen and the first rejected candidate (to judge how safe the choice is)."""
    tokens, all_logits, min_gap = [], [], np.inf
    for n_i in tree:
        idx, val = oracle.topk(logits, n_i + 1 if logits.shape[1] > n_i else n_i)
        if val.shape[1] > n_i:
            gaps = np.concatenate([(val[:, :-1] - val[:, 1:]).ravel()])      # all adjacent gaps among the first n_i + 1
            min_gap = min(min_gap, float(gaps.min()))
        tok = idx[:, :n_i].reshape(-1)
        parent = np.arange(tok.size) // n_i
        hid = oracle.embedding(tok, w["embedding"])
        conv, ssm = conv[:, parent], ssm[:, parent]
        new_conv, new_ssm = [], []
        for l, bw in enumerate(w["blocks"]):
            out, cs, hs = oracle.block_fwd(bw, hid[:, None, :], conv_state_in=conv[l], h0=ssm[l], eps=eps)
            hid = _rb(out[:, 0])
            new_conv.append(_rb(cs))
            new_ssm.append(hs)
        conv, ssm = np.stack(new_conv), np.stack(new_ssm)
        logits = _rb(oracle.linear(_rb(oracle.rmsnorm(hid, w["norm_f"], eps)), w["lm_head"]))
        tokens.append(tok.astype(np.int32))
        all_logits.append(logits)
    return tokens, all_logits, min_gap
