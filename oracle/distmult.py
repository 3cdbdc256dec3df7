"""DistMult link-prediction decoder with shared negatives, forward and backward, in NumPy fp64.
TEST INFRASTRUCTURE ONLY (see the package docstring).

What it follows: the MariusGNN paper names the decoder only (Section 7.1, link prediction: the
encoder's output representations are scored with the DistMult score function; negative samples are
drawn per training edge, 500 of them in Section 7.3) and prints neither the score formula nor the
loss nor the negative-sampling scheme.  The decoder is therefore the textbook one (Yang et al.,
"Embedding entities and relations for learning and inference in knowledge bases", 2015) with the
following readings:

  - score        f(s, r, d) = sum_j h_s[j] * r[j] * h_d[j]
  - negatives    the edges of a batch are cut into chunks of `chunk` consecutive edges; chunk q shares
                 one list of negative nodes neg[q, :].  Corrupting the destination of edge e (chunk q)
                 scores f(src_e, rel_e, neg[q, n]); corrupting the source scores f(neg[q, n], rel_e, dst_e).
  - loss         per edge and per corrupted side, softmax cross-entropy of the positive against that side's
                 negatives:  logsumexp([pos, neg_1 .. neg_Nn]) - pos;  an edge's loss is the sum of its two
                 sides; the batch loss is the plain sum over edges (the caller scales).
  - precision    mode "exact" is fp64 throughout.  Mode "bf16" models the negatives' scores as a
                 matrix-core contraction: the operands q = bf16(fp32(h_a * r)) (a = source for destination
                 corruption, destination for source corruption; the product is formed in fp32 first) and
                 bf16(h_neg) are one bfloat16 term each, products and sums fp64.  The positive's score uses
                 the unrounded fp32 inputs.  Backward differentiates through the rounding as if it were the
                 identity; the softmax probabilities that enter the two backward contractions are device-
                 computed values and therefore two bfloat16 terms (see sage.py on why), the other operand of
                 those contractions is the same bf16 matrix the forward pass used.
"""
from dataclasses import dataclass

import numpy as np

from .sage import bf16_terms, round_bf16


@dataclass
class DistMultState:
    H: np.ndarray          # [n, d] node representations (decoder input)
    R: np.ndarray          # [n_rel, d] relation embeddings
    src: np.ndarray        # [B] row of H per edge source
    rel: np.ndarray        # [B]
    dst: np.ndarray        # [B]
    neg: np.ndarray        # [C, Nn] rows of H, C = ceil(B / chunk)
    chunk: int
    mode: str
    pos: np.ndarray        # [B]
    neg_dst: np.ndarray    # [B, Nn] scores with the destination corrupted
    neg_src: np.ndarray    # [B, Nn] scores with the source corrupted
    lse_dst: np.ndarray    # [B]
    lse_src: np.ndarray    # [B]
    loss: np.ndarray       # [B]
    q_dst: np.ndarray      # [B, d] operand of neg_dst (h_src * r, rounded in bf16 mode)
    q_src: np.ndarray      # [B, d] operand of neg_src (h_dst * r)
    e_neg: np.ndarray      # [C, Nn, d] negatives' rows as used by the contraction


def _logsumexp_with(pos: np.ndarray, negs: np.ndarray) -> np.ndarray:
    m = np.maximum(pos, negs.max(axis=1)) if negs.shape[1] else pos
    return m + np.log(np.exp(pos - m) + np.exp(negs - m[:, None]).sum(axis=1))


def distmult_forward(H, R, src, rel, dst, neg, chunk: int, mode: str = "exact") -> DistMultState:
    assert mode in ("exact", "bf16")
    H32 = np.ascontiguousarray(H, dtype=np.float32)
    R32 = np.ascontiguousarray(R, dtype=np.float32)
    src, rel, dst = (np.asarray(a, dtype=np.int64) for a in (src, rel, dst))
    neg = np.asarray(neg, dtype=np.int64)
    B = len(src)
    C = (B + chunk - 1) // chunk
    assert neg.ndim == 2 and neg.shape[0] == C
    Nn = neg.shape[1]
    Hd, Rd = H32.astype(np.float64), R32.astype(np.float64)
    pos = (Hd[src] * Rd[rel] * Hd[dst]).sum(axis=1)
    if mode == "exact":
        q_dst, q_src, e_neg = Hd[src] * Rd[rel], Hd[dst] * Rd[rel], Hd[neg]
    else:
        q_dst = round_bf16(H32[src] * R32[rel]).astype(np.float64)      # fp32 product, then bf16
        q_src = round_bf16(H32[dst] * R32[rel]).astype(np.float64)
        e_neg = round_bf16(H32[neg]).astype(np.float64)
    neg_dst = np.zeros((B, Nn))
    neg_src = np.zeros((B, Nn))
    for q in range(C):
        lo, hi = q * chunk, min(B, (q + 1) * chunk)
        neg_dst[lo:hi] = q_dst[lo:hi] @ e_neg[q].T
        neg_src[lo:hi] = q_src[lo:hi] @ e_neg[q].T
    lse_dst = _logsumexp_with(pos, neg_dst)
    lse_src = _logsumexp_with(pos, neg_src)
    loss = (lse_dst - pos) + (lse_src - pos)
    return DistMultState(H32, R32, src, rel, dst, neg, chunk, mode, pos, neg_dst, neg_src, lse_dst, lse_src, loss,
                         q_dst, q_src, e_neg)


def distmult_backward(st: DistMultState):
    """Gradients of sum(loss) with respect to H and R."""
    Hd, Rd = st.H.astype(np.float64), st.R.astype(np.float64)
    B, Nn = st.neg_dst.shape
    dH = np.zeros_like(Hd)
    dR = np.zeros_like(Rd)
    p_dst = np.exp(st.neg_dst - st.lse_dst[:, None])
    p_src = np.exp(st.neg_src - st.lse_src[:, None])
    d_pos = (np.exp(st.pos - st.lse_dst) - 1.0) + (np.exp(st.pos - st.lse_src) - 1.0)
    if st.mode == "bf16":
        p_dst, p_src = bf16_terms(p_dst, 2), bf16_terms(p_src, 2)
    dq_dst = np.zeros_like(st.q_dst)
    dq_src = np.zeros_like(st.q_src)
    for q in range(st.neg.shape[0]):
        lo, hi = q * st.chunk, min(B, (q + 1) * st.chunk)
        dq_dst[lo:hi] = p_dst[lo:hi] @ st.e_neg[q]
        dq_src[lo:hi] = p_src[lo:hi] @ st.e_neg[q]
        d_e = p_dst[lo:hi].T @ st.q_dst[lo:hi] + p_src[lo:hi].T @ st.q_src[lo:hi]      # [Nn, d]
        np.add.at(dH, st.neg[q], d_e)
    hs, hd, r = Hd[st.src], Hd[st.dst], Rd[st.rel]
    np.add.at(dH, st.src, d_pos[:, None] * (r * hd) + dq_dst * r)
    np.add.at(dH, st.dst, d_pos[:, None] * (r * hs) + dq_src * r)
    np.add.at(dR, st.rel, d_pos[:, None] * (hs * hd) + dq_dst * hs + dq_src * hd)
    return dH, dR
