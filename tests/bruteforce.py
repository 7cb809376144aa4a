"""Scalar-loop transformer forward, written independently of oracle/ for tiny sizes.

Only Python floats, `math`, lists and for-loops: no numpy arithmetic, no shared
helper with the oracle.  It follows the same reading of the paper (Method,
"Model-level optimization": stacked transformer layers with multi-head
self-attention and feed-forward blocks, tied trimmed output table) so that an
index, sign or transposition mistake in the oracle disagrees with it.
"""
import math


def _ln(row, g, b, eps):
    n = len(row)
    mu = sum(row) / n
    var = sum((v - mu) * (v - mu) for v in row) / n
    inv = 1.0 / math.sqrt(var + eps)
    return [g[i] * ((row[i] - mu) * inv) + b[i] for i in range(n)]


def _gelu(a):
    return a * 0.5 * (1.0 + math.erf(a / math.sqrt(2.0)))


def _linear(x, W, b):
    # W is [out][in]
    return [sum(W[o][i] * x[i] for i in range(len(x))) + b[o] for o in range(len(W))]


def forward(weights, n_heads, eps, ids, L):
    """weights: nested python lists (floats). Returns final hidden rows [n][d]."""
    E, Ep = weights["tok_emb"], weights["pos_emb"]
    n = len(ids)
    d = len(E[0])
    dh = d // n_heads
    X = []
    Et = weights.get("type_emb")        # optional: row 0 for prompt positions, row 1 for generated ones
    for i in range(n):
        row = [E[ids[i]][c] + Ep[i][c] for c in range(d)]
        if Et is not None:
            seg = Et[0] if i < L else Et[1]
            row = [row[c] + seg[c] for c in range(d)]
        X.append(_ln(row, weights["emb_ln_g"], weights["emb_ln_b"], eps))
    for lw in weights["layers"]:
        q, k, v = [], [], []
        for i in range(n):
            qkv = _linear(X[i], lw["wqkv"], lw["bqkv"])
            q.append(qkv[0:d]); k.append(qkv[d:2 * d]); v.append(qkv[2 * d:3 * d])
        O = [[0.0] * d for _ in range(n)]
        for h in range(n_heads):
            c0 = h * dh
            for i in range(n):
                keys = [j for j in range(n) if (j < L or j <= i)]
                s = {}
                for j in keys:
                    s[j] = sum(q[i][c0 + c] * k[j][c0 + c] for c in range(dh)) / math.sqrt(dh)
                m = max(s.values())
                den = sum(math.exp(s[j] - m) for j in keys)
                for j in keys:
                    pj = math.exp(s[j] - m) / den
                    for c in range(dh):
                        O[i][c0 + c] += pj * v[j][c0 + c]
        X1 = []
        for i in range(n):
            a = _linear(O[i], lw["wo"], lw["bo"])
            X1.append(_ln([X[i][c] + a[c] for c in range(d)], lw["ln1_g"], lw["ln1_b"], eps))
        X2 = []
        for i in range(n):
            g = [_gelu(t) for t in _linear(X1[i], lw["w1"], lw["b1"])]
            y = _linear(g, lw["w2"], lw["b2"])
            X2.append(_ln([X1[i][c] + y[c] for c in range(d)], lw["ln2_g"], lw["ln2_b"], eps))
        X = X2
    return X


def generate(weights, n_heads, eps, prompt, n_gen, kept_ids):
    """Greedy generation by full recompute; returns (tokens in trimmed index space, logits rows)."""
    E = weights["tok_emb"]
    L = len(prompt)
    seq = list(prompt)
    toks, logits = [], []
    for _ in range(n_gen):
        H = forward(weights, n_heads, eps, seq, L)
        h = H[-1]
        if weights.get("head_w") is not None:       # optional output head: LN(gelu(W h + b))
            u = [_gelu(t) for t in _linear(h, weights["head_w"], weights["head_b"])]
            h = _ln(u, weights["head_ln_g"], weights["head_ln_b"], eps)
        z = [sum(E[v][c] * h[c] for c in range(len(h))) for v in kept_ids]
        if weights.get("out_bias") is not None:     # optional bias, indexed by FULL vocabulary id
            z = [z[t] + weights["out_bias"][kept_ids[t]] for t in range(len(kept_ids))]
        best = 0
        for kk in range(1, len(z)):
            if z[kk] > z[best]:
                best = kk
        toks.append(best)
        logits.append(z)
        seq.append(kept_ids[best])
    return toks, logits


def to_lists(weights):
    """numpy weight dict -> nested python float lists."""
    def c(a):
        return a.astype("float64").tolist()
    out = {k: c(v) for k, v in weights.items() if k != "layers"}
    out["layers"] = [{k: c(v) for k, v in lw.items()} for lw in weights["layers"]]
    return out
