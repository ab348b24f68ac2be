"""Float64 oracle of the attention inside the action expert and the language expert.

Test infrastructure only (see the package docstring).

What is computed (paper Sec. 3.1, Eq. 1-2; App. A.1, Eq. 5-6):

* Every expert conditions on the prefill cache K_t of the frame the request was
  created in (Eq. 2), so every query sees all P prefix tokens.
* The language expert is autoregressive (Eq. 5): the query of own token p sees
  own tokens 0..p (its own key/value was appended in the same pass, App. A.2
  "K_t' extends K_t with KVs from newly decoded tokens").
* The action expert produces the whole chunk jointly (Eq. 6): each chunk query
  sees every chunk token, in both directions.
* Nothing else is visible.  In particular the action expert's view is the
  read-only prefill cache (Sec. 1, "heterogeneous expert KV semantics"), so no
  language-side append may ever enter it.

Sharing and batching are claimed lossless by the paper (Sec. 1: identical KV
entries per task; Sec. 3.2), hence the oracle is the plain definition with no
paging, no sharing and no batching:

    s_j      = scale * <q[r,h,:], k_j>          one KV head serves all 8 query heads
    O[r,h,:] = sum_j softmax_j(s) * v_j
    LSE[r,h] = log sum_j exp(s_j)               natural log

Inputs are bf16 bit patterns (uint16); they are widened exactly to float64 here.
"""
import numpy as np

ACTION = 0
DECODE = 1


def widen_bf16(bits):
    """Exact bf16 -> float64: a bf16 is the upper half of an IEEE float32."""
    bits = np.asarray(bits)
    if bits.dtype != np.uint16:
        raise TypeError("bf16 bit patterns must be uint16")
    as_f32 = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    with np.errstate(invalid="ignore"):         # signalling-NaN patterns widen to NaN
        return as_f32.astype(np.float64)


def visible_counts(kind, n_prefix, n_own, m_new, r):
    """Number of visible prefix tokens and own tokens for new query r (0-based).

    The m_new queries are the last m_new of the stream's n_own own tokens, so
    query r sits at own position p = n_own - m_new + r.
    """
    if not (0 <= r < m_new <= n_own):
        raise ValueError("query index out of range")
    p = n_own - m_new + r
    if kind == ACTION:
        return n_prefix, n_own
    if kind == DECODE:
        return n_prefix, p + 1
    raise ValueError("unknown kind")


def softmax_attend(q, k, v, scale):
    """One query token (all heads) over an explicit key/value set.

    q: [H, d] float64, k/v: [n, d] float64, n >= 1.  Returns (O [H, d], LSE [H]).
    """
    s = scale * (q @ k.T)                       # [H, n]
    mx = s.max(axis=1, keepdims=True)
    e = np.exp(s - mx)
    z = e.sum(axis=1, keepdims=True)
    o = (e / z) @ v
    lse = (mx + np.log(z))[:, 0]
    return o, lse


def attend_item(kind, q_bits, kp_bits, vp_bits, ko_bits, vo_bits, scale):
    """Attention output of one batch item for one layer.

    q_bits  [m, H, d] uint16   the m new queries of the item
    kp/vp   [P, d]    uint16   logical prefix of the stream's birth frame (P may be 0)
    ko/vo   [n, d]    uint16   all own tokens of the stream, the new ones included
    Returns O [m, H, d] float64 and LSE [m, H] float64.
    """
    q = widen_bf16(q_bits)
    kp, vp = widen_bf16(kp_bits), widen_bf16(vp_bits)
    ko, vo = widen_bf16(ko_bits), widen_bf16(vo_bits)
    m = q.shape[0]
    n_prefix, n_own = kp.shape[0], ko.shape[0]
    out = np.empty(q.shape, dtype=np.float64)
    lse = np.empty(q.shape[:2], dtype=np.float64)
    for r in range(m):
        vis_p, vis_o = visible_counts(kind, n_prefix, n_own, m, r)
        k = np.concatenate([kp[:vis_p], ko[:vis_o]], axis=0)
        v = np.concatenate([vp[:vis_p], vo[:vis_o]], axis=0)
        out[r], lse[r] = softmax_attend(q[r], k, v, scale)
    return out, lse


def merge_partials(parts):
    """Combine attention results over disjoint key sets into the result over their union.

    parts: list of (O, LSE) computed over disjoint, jointly exhaustive key sets.
    Identity: LSE = log sum_i exp(LSE_i), O = sum_i exp(LSE_i - LSE) * O_i.
    Stated here because it is what any split-KV evaluation must satisfy.
    """
    lses = np.stack([p[1] for p in parts], axis=0)
    mx = lses.max(axis=0)
    w = np.exp(lses - mx)
    z = w.sum(axis=0)
    o = sum(wi[..., None] * p[0] for wi, p in zip(w, parts)) / z[..., None]
    return o, mx + np.log(z)
