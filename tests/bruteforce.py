"""Per-vertex recursive evaluation of a GNN on a small graph (vertex-wise
inference, Sec. 1.1 of the paper): h^l_v is computed from the h^{l-1} of v's
in-neighbours, each of which is computed the same way, down to the features.
Plain Python loops over an adjacency dict; shares nothing with the oracle's
matrix formulation. Only usable on tiny graphs."""
import numpy as np


def in_lists(n, src, dst):
    nbrs = {v: [] for v in range(n)}
    for s, d in zip(list(src), list(dst)):
        nbrs[int(d)].append(int(s))
    return nbrs


def in_weights(src, dst, w):
    """{(u, v): alpha_uv} for the weighted sum."""
    return {(int(s), int(d)): float(x) for s, d, x in zip(list(src), list(dst), list(w))}


def embed(v, l, model, feats, nbrs, alive, memo, alpha=None):
    """h^l_v as float64 vector; alpha: edge weights for layers that aggregate by weighted sum."""
    key = (v, l)
    if key in memo:
        return memo[key]
    if not alive[v]:
        width = model[l - 1]["d_out"] if l else feats.shape[1]
        res = np.zeros(width)
    elif l == 0:
        res = np.array(feats[v], dtype=np.float64)
    else:
        lay = model[l - 1]
        if lay["agg"] == "attn":                      # Eq. (3) with plain loops
            import math
            W0 = np.array(lay["W0"], dtype=np.float64)
            att = np.array(lay["att"], dtype=np.float64)
            n_out = lay["d_out"]

            def proj(x):
                out = np.zeros(n_out)
                for k in range(lay["d_in"]):
                    out = out + x[k] * W0[k]
                return out
            p_v = proj(embed(v, l - 1, model, feats, nbrs, alive, memo, alpha))
            t_v = sum(att[n_out + k] * p_v[k] for k in range(n_out))
            num, den = np.zeros(n_out), 0.0
            for u in nbrs[v]:
                p_u = proj(embed(u, l - 1, model, feats, nbrs, alive, memo, alpha))
                z = sum(att[k] * p_u[k] for k in range(n_out)) + t_v
                z = z if z > 0 else 0.2 * z
                num = num + math.exp(z) * p_u
                den = den + math.exp(z)
            z = np.array(lay["b0"], dtype=np.float64) + (num / den if den > 0 else 0.0)
            if lay["act_out"] == "relu":
                z = np.where(z > 0, z, 0.0)
            memo[key] = z
            return z
        acc = np.zeros(lay["d_in"])
        first = True
        for u in nbrs[v]:
            term = embed(u, l - 1, model, feats, nbrs, alive, memo, alpha)
            if lay["agg"] in ("max", "min"):          # element by element, plain comparisons
                if first:
                    acc = np.array(term, dtype=np.float64)
                else:
                    for k in range(lay["d_in"]):
                        if (term[k] > acc[k]) if lay["agg"] == "max" else (term[k] < acc[k]):
                            acc[k] = term[k]
                first = False
                continue
            acc = acc + (alpha[(u, v)] * term if lay["agg"] == "wsum" else term)
        if lay["agg"] == "mean" and len(nbrs[v]) > 0:
            acc = acc / len(nbrs[v])
        own = embed(v, l - 1, model, feats, nbrs, alive, memo, alpha)
        W0 = np.array(lay["W0"], dtype=np.float64)
        b0 = np.array(lay["b0"], dtype=np.float64)
        z = np.array(b0)
        if lay["self"] == "none":
            for k in range(lay["d_in"]):
                z = z + acc[k] * W0[k]
        elif lay["self"] == "concat":
            for k in range(lay["d_in"]):
                z = z + own[k] * W0[k] + acc[k] * W0[lay["d_in"] + k]
        else:
            r = (1.0 + lay["eps"]) * own + acc
            for k in range(lay["d_in"]):
                z = z + r[k] * W0[k]
        if lay["d_hidden"]:
            if lay["act_inner"] == "relu":
                z = np.where(z > 0, z, 0.0)
            W1 = np.array(lay["W1"], dtype=np.float64)
            z2 = np.array(lay["b1"], dtype=np.float64)
            for k in range(lay["d_hidden"]):
                z2 = z2 + z[k] * W1[k]
            z = z2
        if lay["act_out"] == "relu":
            z = np.where(z > 0, z, 0.0)
        res = z
    memo[key] = res
    return res
