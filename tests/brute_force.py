"""Brute-force, loop-by-loop versions of the attention kinds, LayerNorm and Linear.

Pure Python floats and ``math`` only, no numpy arithmetic: an implementation so
different from the oracle's batched matmuls that a shared mistake is implausible.
Only usable at tiny sizes.  Written from the definitions (section 2.2 of the paper:
which tokens each attention kind relates; softmax attention as usually defined)."""
import math


def softmax_attention_rows(Q, K, V, n_valid=None):
    """Q [Lq][dh], K,V [Lk][dh] as nested lists -> O [Lq][dh]."""
    Lq, Lk, dh = len(Q), len(K), len(Q[0])
    nk = Lk if n_valid is None else n_valid
    out = []
    for i in range(Lq):
        logits = []
        for j in range(nk):
            acc = 0.0
            for d in range(dh):
                acc += Q[i][d] * K[j][d]
            logits.append(acc / math.sqrt(dh))
        mx = max(logits)
        w = [math.exp(l - mx) for l in logits]
        z = sum(w)
        row = []
        for d in range(dh):
            acc = 0.0
            for j in range(nk):
                acc += (w[j] / z) * V[j][d]
            row.append(acc)
        out.append(row)
    return out


def spatial(q, k, v):
    """q,k,v nested [B][T][S][H][dh]."""
    B, T, S, H = len(q), len(q[0]), len(q[0][0]), len(q[0][0][0])
    o = [[[[None] * H for _ in range(S)] for _ in range(T)] for _ in range(B)]
    for b in range(B):
        for t in range(T):
            for h in range(H):
                Q = [q[b][t][s][h] for s in range(S)]
                K = [k[b][t][s][h] for s in range(S)]
                V = [v[b][t][s][h] for s in range(S)]
                O = softmax_attention_rows(Q, K, V)
                for s in range(S):
                    o[b][t][s][h] = O[s]
    return o


def temporal(q, k, v):
    B, T, S, H = len(q), len(q[0]), len(q[0][0]), len(q[0][0][0])
    o = [[[[None] * H for _ in range(S)] for _ in range(T)] for _ in range(B)]
    for b in range(B):
        for s in range(S):
            for h in range(H):
                Q = [q[b][t][s][h] for t in range(T)]
                K = [k[b][t][s][h] for t in range(T)]
                V = [v[b][t][s][h] for t in range(T)]
                O = softmax_attention_rows(Q, K, V)
                for t in range(T):
                    o[b][t][s][h] = O[t]
    return o


def cross(q, k, v, valid_len):
    """q [B][L][H][dh], k,v [B][Ly][H][dh]."""
    B, L, H = len(q), len(q[0]), len(q[0][0])
    Ly = len(k[0])
    o = [[[None] * H for _ in range(L)] for _ in range(B)]
    for b in range(B):
        for h in range(H):
            Q = [q[b][i][h] for i in range(L)]
            K = [k[b][j][h] for j in range(Ly)]
            V = [v[b][j][h] for j in range(Ly)]
            O = softmax_attention_rows(Q, K, V, None if valid_len is None else valid_len[b])
            for i in range(L):
                o[b][i][h] = O[i]
    return o


def layer_norm_row(u, eps):
    n = len(u)
    mu = sum(u) / n
    var = sum((a - mu) * (a - mu) for a in u) / n
    return [(a - mu) / math.sqrt(var + eps) for a in u]


def linear_row(u, W, b):
    """u [in], W [out][in], b [out]."""
    return [sum(W[o][i] * u[i] for i in range(len(u))) + b[o] for o in range(len(W))]


def rms_norm_row(u, g, eps):
    """u, g lists -> u / sqrt(mean(u^2) + eps) * g, element by element."""
    ms = 0.0
    for a in u:
        ms += a * a
    ms /= len(u)
    return [a / math.sqrt(ms + eps) * w for a, w in zip(u, g)]


def rotary_row(u, pos, theta=10000.0):
    """Rotary embedding of one vector, written as complex multiplication: the pair
    (u[2i], u[2i+1]) read as the complex number u[2i] + 1j u[2i+1] is multiplied by
    exp(1j pos theta^(-2i/d))."""
    import cmath
    d = len(u)
    out = []
    for i in range(d // 2):
        z = complex(u[2 * i], u[2 * i + 1]) * cmath.exp(1j * pos * theta ** (-2.0 * i / d))
        out += [z.real, z.imag]
    return out
