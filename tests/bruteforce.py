"""Element-by-element float64 transformer for tiny shapes (pure Python loops).

An independent pin for the oracle: it walks one sequence token by token with scalar
arithmetic from the `math` module, shares nothing with oracle/ and uses no matrix
routine.  Weights are nested lists or arrays indexed [out][in]."""
import math


def _rmsnorm(x, g, eps):
    ms = sum(v * v for v in x) / len(x)
    r = 1.0 / math.sqrt(ms + eps)
    return [x[i] * r * float(g[i]) for i in range(len(x))]


def _matvec(w, x):
    return [sum(float(w[n][k]) * x[k] for k in range(len(x))) for n in range(len(w))]


def _rope(vec, pos, base):
    hd = len(vec)
    half = hd // 2
    out = [0.0] * hd
    for i in range(half):
        ang = pos * base ** (-2.0 * i / hd)
        c, s = math.cos(ang), math.sin(ang)
        out[i] = vec[i] * c - vec[i + half] * s
        out[i + half] = vec[i + half] * c + vec[i] * s
    return out


def forward(cfg, w, tokens):
    """Logits [T][V] of one sequence.  cfg: dict with the usual keys."""
    L, d = cfg["n_layers"], cfg["d_model"]
    Hq, Hkv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    G = Hq // Hkv
    eps, base = cfg["rms_eps"], cfg["rope_base"]
    kc = [[] for _ in range(L)]      # kc[l][pos][kvh] -> list hd
    vc = [[] for _ in range(L)]
    logits = []
    for pos, tok in enumerate(tokens):
        x = [float(v) for v in w["embed"][tok]]
        for l in range(L):
            lw = w["layers"][l]
            h = _rmsnorm(x, lw["attn_norm"], eps)
            q = _matvec(lw["wq"], h)
            k = _matvec(lw["wk"], h)
            v = _matvec(lw["wv"], h)
            qh = [_rope(q[a * hd:(a + 1) * hd], pos, base) for a in range(Hq)]
            kh = [_rope(k[c * hd:(c + 1) * hd], pos, base) for c in range(Hkv)]
            vh = [v[c * hd:(c + 1) * hd] for c in range(Hkv)]
            kc[l].append(kh)
            vc[l].append(vh)
            o = []
            for a in range(Hq):
                c = a // G
                s = [sum(qh[a][i] * kc[l][j][c][i] for i in range(hd)) / math.sqrt(hd)
                     for j in range(pos + 1)]
                m = max(s)
                e = [math.exp(t - m) for t in s]
                z = sum(e)
                for i in range(hd):
                    o.append(sum(e[j] / z * vc[l][j][c][i] for j in range(pos + 1)))
            att = _matvec(lw["wo"], o)
            x = [x[i] + att[i] for i in range(d)]
            h2 = _rmsnorm(x, lw["ffn_norm"], eps)
            gate = _matvec(lw["w_gate"], h2)
            up = _matvec(lw["w_up"], h2)
            act = [gate[i] / (1.0 + math.exp(-gate[i])) * up[i] for i in range(len(gate))]
            dn = _matvec(lw["w_down"], act)
            x = [x[i] + dn[i] for i in range(d)]
        hf = _rmsnorm(x, w["final_norm"], eps)
        logits.append(_matvec(w["lm_head"], hf))
    return logits
