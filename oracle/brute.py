"""Pure-Python brute force of the attention equation (paper Section 2.1) for one request.

TEST INFRASTRUCTURE ONLY.  It exists to pin the C oracle on tiny inputs: nested
loops over Python floats and ``math.exp``, nothing vectorised, nothing shared
with the C oracle or with the GPU code.
"""
import math


def attention_one_request(q, k, v, scale, n_q_heads, n_kv_heads):
    """softmax(q k^T * scale) v with bottom-right causal alignment.

    q: [q_len][Hq][d], k and v: [kv_len][Hkv][d] as nested sequences of floats.
    Local query row i sits at absolute position kv_len - q_len + i and sees keys
    0..that position (Sections 2.1 and 5.2: a chunk reads the cache of all prior
    chunks plus itself; a decode is q_len == 1).  Query head h uses K/V head
    h // (Hq // Hkv) (Section 2.1).
    """
    q_len, kv_len = len(q), len(k)
    d = len(q[0][0])
    group = n_q_heads // n_kv_heads
    out = []
    for i in range(q_len):
        last = kv_len - q_len + i
        row = []
        for h in range(n_q_heads):
            kvh = h // group
            scores = []
            for j in range(last + 1):
                acc = 0.0
                for c in range(d):
                    acc += float(q[i][h][c]) * float(k[j][kvh][c])
                scores.append(acc * scale)
            top = max(scores)
            weights = [math.exp(s - top) for s in scores]
            total = sum(weights)
            vec = []
            for c in range(d):
                acc = 0.0
                for j in range(last + 1):
                    acc += weights[j] * float(v[j][kvh][c])
                vec.append(acc / total)
            row.append(vec)
        out.append(row)
    return out
