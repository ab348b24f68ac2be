"""Pure-Python (no numpy arithmetic) evaluation of the same attention definition.

Test infrastructure only.  Written independently of oracle.attention so that a
slip in either (a dropped term, a wrong bound of the visible set, a transposed
operand) shows up as a disagreement on tiny inputs.  Visibility follows the
paper's Eq. 2, Eq. 5 and Eq. 6: prefix always, own history causally for the
language expert, the whole chunk for the action expert.
"""
import math
import struct

ACTION = 0
DECODE = 1


def bf16_to_float(bits):
    """One bf16 bit pattern (int) to a Python float, via the float32 it prefixes."""
    return struct.unpack("<f", struct.pack("<I", (int(bits) & 0xFFFF) << 16))[0]


def attend_item_loops(kind, q_bits, kp_bits, vp_bits, ko_bits, vo_bits, scale):
    """Nested lists in, nested lists out; shapes as in oracle.attention.attend_item."""
    m = len(q_bits)
    heads = len(q_bits[0])
    d = len(q_bits[0][0])
    n_prefix = len(kp_bits)
    n_own = len(ko_bits)
    out = [[[0.0] * d for _ in range(heads)] for _ in range(m)]
    lse = [[0.0] * heads for _ in range(m)]
    for r in range(m):
        pos = n_own - m + r
        keys = [(kp_bits[j], vp_bits[j]) for j in range(n_prefix)]
        for j in range(n_own):
            if kind == ACTION or j <= pos:
                keys.append((ko_bits[j], vo_bits[j]))
        for h in range(heads):
            logits = []
            for kb, _ in keys:
                acc = 0.0
                for c in range(d):
                    acc += bf16_to_float(q_bits[r][h][c]) * bf16_to_float(kb[c])
                logits.append(scale * acc)
            top = max(logits)
            weights = [math.exp(s - top) for s in logits]
            total = math.fsum(weights)
            for c in range(d):
                out[r][h][c] = math.fsum(
                    w * bf16_to_float(vb[c]) for w, (_, vb) in zip(weights, keys)) / total
            lse[r][h] = top + math.log(total)
    return out, lse
