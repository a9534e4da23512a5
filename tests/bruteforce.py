"""Pure-Python loop versions of the layer's pieces, for tiny shapes only.

Written index by index from the definitions (no numpy broadcasting, no matmul), so that a
transposed operand, a wrong head slice or a dropped term in the vectorised oracle shows up.
"""
import math


def matmul_nt(X, W, b):
    """Y[t][o] = sum_i X[t][i] * W[o][i] + b[o]"""
    T, I, O = len(X), len(X[0]), len(W)
    return [[sum(X[t][i] * W[o][i] for i in range(I)) + b[o] for o in range(O)] for t in range(T)]


def layer_norm(X, gamma, beta, eps):
    out = []
    for row in X:
        n = len(row)
        mu = sum(row) / n
        var = sum((r - mu) ** 2 for r in row) / n
        out.append([gamma[h] * (row[h] - mu) / math.sqrt(var + eps) + beta[h] for h in range(n)])
    return out


def gelu(z):
    return 0.5 * z * (1.0 + math.erf(z / math.sqrt(2.0)))


def attention(qkv, S, H, A, causal):
    """qkv: [S][3H] for one sample.  Returns O [S][H]."""
    d = H // A
    O = [[0.0] * H for _ in range(S)]
    for a in range(A):
        for s in range(S):
            last = s if causal else S - 1
            z = []
            for t in range(last + 1):
                z.append(sum(qkv[s][a * d + e] * qkv[t][H + a * d + e] for e in range(d)) / math.sqrt(d))
            zmax = max(z)
            w = [math.exp(zi - zmax) for zi in z]
            tot = sum(w)
            for e in range(d):
                O[s][a * d + e] = sum(w[t] / tot * qkv[t][2 * H + a * d + e] for t in range(last + 1))
    return O


def layer_fwd(p, X, S, H, F, A, causal, eps):
    """p: dict of nested lists; X: [m*S][H] with samples stacked.  Returns Y [m*S][H]."""
    m = len(X) // S
    U = layer_norm(X, p["ln1_g"], p["ln1_b"], eps)
    QKV = matmul_nt(U, p["w_qkv"], p["b_qkv"])
    O = []
    for n in range(m):
        O += attention(QKV[n * S:(n + 1) * S], S, H, A, causal)
    proj = matmul_nt(O, p["w_o"], p["b_o"])
    X1 = [[X[t][h] + proj[t][h] for h in range(H)] for t in range(len(X))]
    U2 = layer_norm(X1, p["ln2_g"], p["ln2_b"], eps)
    Z = matmul_nt(U2, p["w_fc1"], p["b_fc1"])
    Hh = [[gelu(z) for z in row] for row in Z]
    out = matmul_nt(Hh, p["w_fc2"], p["b_fc2"])
    return [[X1[t][h] + out[t][h] for h in range(H)] for t in range(len(X))]
