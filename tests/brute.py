"""Pure-Python re-derivation of the hot path, used only to pin the oracle.

Scalar loops over Python floats (which are IEEE doubles), math.exp, no numpy
arithmetic and no code shared with oracle/: a second, independent writing of
Section 4.1 of the paper.  Only usable on tiny inputs.
"""
import math
import struct


def _bf16(bits):
    return struct.unpack("<f", struct.pack("<I", int(bits) << 16))[0]


def _e4m3(code):
    code = int(code)
    s = -1.0 if code >= 128 else 1.0
    e = (code // 8) % 16
    m = code % 8
    if e == 15 and m == 7:
        return float("nan")
    if e == 0:
        return s * m * 2.0 ** -9
    return s * (8 + m) * 2.0 ** (e - 10)


def _elem(x, dtype):
    if dtype == "f32":
        return float(x)
    if dtype == "bf16":
        return _bf16(x)
    return _e4m3(x)


def kv_row(w, which, b, t, g):
    page = int(w.block_table[b][t // w.P])
    slot = t % w.P
    pool = w.k_pool if which == "k" else w.v_pool
    row = [_elem(x, w.kv_dtype) for x in pool[page][g][slot]]
    if w.kv_dtype == "fp8_e4m3":
        sc = float((w.k_scale if which == "k" else w.v_scale)[page][g])
        row = [x * sc for x in row]
    return row


def verify(w):
    n_q, G = w.spec_k + 1, w.Hq // w.Hkv
    out = [[[None] * w.Hq for _ in range(n_q)] for _ in range(w.B)]
    lse = [[[None] * w.Hq for _ in range(n_q)] for _ in range(w.B)]
    scores = [[None] * w.Hkv for _ in range(w.B)]
    for b in range(w.B):
        L = int(w.seq_lens[b])
        for g in range(w.Hkv):
            K = [kv_row(w, "k", b, t, g) for t in range(L)]
            V = [kv_row(w, "v", b, t, g) for t in range(L)]
            acc = [0.0] * L
            for i in range(n_q):
                last = L - n_q + i
                for h in range(g * G, (g + 1) * G):
                    q = [_elem(x, w.q_dtype) for x in w.q[b][i][h]]
                    if last < 0:                      # the query sees no token: nothing to normalise
                        out[b][i][h] = [0.0] * w.D
                        lse[b][i][h] = -math.inf
                        continue
                    s = []
                    for t in range(last + 1):
                        d = 0.0
                        for a, c in zip(q, K[t]):
                            d += a * c
                        s.append(d * w.sm_scale)
                    mx = max(s)
                    den = 0.0
                    for x in s:
                        den += math.exp(x - mx)
                    o = [0.0] * w.D
                    for t in range(last + 1):
                        p = math.exp(s[t] - mx) / den
                        acc[t] += p
                        for d in range(w.D):
                            o[d] += p * V[t][d]
                    out[b][i][h] = o
                    lse[b][i][h] = mx + math.log(den)
            scores[b][g] = [a / (n_q * G) for a in acc]
    return out, lse, scores


def topk(score_row, k):
    """k largest by repeated selection; ties to the lower position."""
    left = list(range(len(score_row)))
    chosen = []
    for _ in range(min(k, len(score_row))):
        best = left[0]
        for t in left:
            if score_row[t] > score_row[best]:
                best = t
        chosen.append(best)
        left.remove(best)
    return sorted(chosen)


def sparse(w, indices, counts):
    G = w.Hq // w.Hkv
    out = [[None] * w.Hq for _ in range(w.B)]
    lse = [[None] * w.Hq for _ in range(w.B)]
    for b in range(w.B):
        n = int(counts[b])
        for g in range(w.Hkv):
            sel = [int(x) for x in indices[b][g][:n]]
            K = [kv_row(w, "k", b, t, g) for t in sel]
            V = [kv_row(w, "v", b, t, g) for t in sel]
            for h in range(g * G, (g + 1) * G):
                q = [_elem(x, w.q_dtype) for x in w.q_draft[b][h]]
                s = [w.sm_scale * sum(a * c for a, c in zip(q, row)) for row in K]
                mx = max(s)
                den = sum(math.exp(x - mx) for x in s)
                o = [0.0] * w.D
                for j, x in enumerate(s):
                    p = math.exp(x - mx) / den
                    for d in range(w.D):
                        o[d] += p * V[j][d]
                out[b][h] = o
                lse[b][h] = mx + math.log(den)
    return out, lse
