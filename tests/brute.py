"""A deliberately naive scalar evaluator of the stage, written straight from the operator
definitions with Python loops and Python floats (double precision). It exists only to pin
the numpy oracle on tiny inputs; it shares nothing with it."""
import math


def zeros(*shape):
    if len(shape) == 1:
        return [0.0] * shape[0]
    return [zeros(*shape[1:]) for _ in range(shape[0])]


def conv3x3(x, w, b, stride=1):
    N, Cin, H, W = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0])
    Cout = len(w)
    Ho, Wo = H // stride, W // stride
    y = zeros(N, Cout, Ho, Wo)
    for n in range(N):
        for o in range(Cout):
            for i in range(Ho):
                for j in range(Wo):
                    acc = b[o]
                    for c in range(Cin):
                        for a in range(3):
                            for e in range(3):
                                ii = stride * i + a - 1
                                jj = stride * j + e - 1
                                if 0 <= ii < H and 0 <= jj < W:
                                    acc += w[o][c][a][e] * x[n][c][ii][jj]
                    y[n][o][i][j] = acc
    return y


def group_norm_silu(x, gamma, beta, G, eps, act=True):
    N, C, H, W = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0])
    cg = C // G
    y = zeros(N, C, H, W)
    for n in range(N):
        for g in range(G):
            vals = [x[n][c][i][j] for c in range(g * cg, (g + 1) * cg) for i in range(H) for j in range(W)]
            mu = sum(vals) / len(vals)
            var = sum((v - mu) ** 2 for v in vals) / len(vals)
            r = 1.0 / math.sqrt(var + eps)
            for c in range(g * cg, (g + 1) * cg):
                for i in range(H):
                    for j in range(W):
                        t = (x[n][c][i][j] - mu) * r * gamma[c] + beta[c]
                        y[n][c][i][j] = t / (1.0 + math.exp(-t)) if act else t
    return y


def attn_rows(X, wq, wk, wv, wo, bo, heads):
    """X: list of L rows of C floats -> list of L rows of C floats."""
    L, C = len(X), len(X[0])
    d = C // heads

    def lin(row, w):
        return [sum(w[o][c] * row[c] for c in range(C)) for o in range(C)]

    Q = [lin(r, wq) for r in X]
    K = [lin(r, wk) for r in X]
    V = [lin(r, wv) for r in X]
    O = zeros(L, C)
    for hd in range(heads):
        for i in range(L):
            s = [sum(Q[i][hd * d + k] * K[j][hd * d + k] for k in range(d)) / math.sqrt(d) for j in range(L)]
            m = max(s)
            e = [math.exp(v - m) for v in s]
            z = sum(e)
            for k in range(d):
                O[i][hd * d + k] = sum(e[j] / z * V[j][hd * d + k] for j in range(L))
    return [[bo[o] + sum(wo[o][c] * O[i][c] for c in range(C)) for o in range(C)] for i in range(L)]


def attn_core(Q, K, V, heads):
    """Q: Lq rows, K and V: L rows, of C floats each -> Lq rows of C floats: per head, every query's
    scores against all keys divided by sqrt(d), softmax over the keys, weighted sum of the values."""
    Lq, L, C = len(Q), len(K), len(Q[0])
    d = C // heads
    O = zeros(Lq, C)
    for hd in range(heads):
        for i in range(Lq):
            s = [sum(Q[i][hd * d + k] * K[j][hd * d + k] for k in range(d)) / math.sqrt(d) for j in range(L)]
            m = max(s)
            e = [math.exp(v - m) for v in s]
            z = sum(e)
            for k in range(d):
                O[i][hd * d + k] = sum(e[j] * V[j][hd * d + k] for j in range(L)) / z
    return O


def stage(cfg, w, x, deep_in=None):
    """x: nested list [N][C_lat][H][W]. Returns (eps, deep). If deep_in is given it is used
    (cached step) instead of running the deep branch (full step)."""
    N, H, W, C, G = cfg.B * cfg.F, cfg.H, cfg.W, cfg.C, cfg.groups
    h = conv3x3(x, w["conv_in.w"], w["conv_in.b"])
    for r in range(cfg.n_res):
        t = conv3x3(group_norm_silu(h, w[f"res{r}.gn_g"], w[f"res{r}.gn_b"], G, cfg.gn_eps),
                    w[f"res{r}.w"], w[f"res{r}.b"])
        h = [[[[h[n][c][i][j] + t[n][c][i][j] for j in range(W)] for i in range(H)] for c in range(C)] for n in range(N)]
    # spatial attention: tokens are positions of one frame
    g = group_norm_silu(h, w["sattn.gn_g"], w["sattn.gn_b"], G, cfg.gn_eps, act=False)
    for n in range(N):
        X = [[g[n][c][i][j] for c in range(C)] for i in range(H) for j in range(W)]
        Y = attn_rows(X, w["sattn.wq"], w["sattn.wk"], w["sattn.wv"], w["sattn.wo"], w["sattn.bo"], cfg.heads)
        for i in range(H):
            for j in range(W):
                for c in range(C):
                    h[n][c][i][j] += Y[i * W + j][c]
    # temporal attention: tokens are the frames of one (batch, position)
    g = group_norm_silu(h, w["tattn.gn_g"], w["tattn.gn_b"], G, cfg.gn_eps, act=False)
    for bb in range(cfg.B):
        for i in range(H):
            for j in range(W):
                X = [[g[bb * cfg.F + f][c][i][j] for c in range(C)] for f in range(cfg.F)]
                Y = attn_rows(X, w["tattn.wq"], w["tattn.wk"], w["tattn.wv"], w["tattn.wo"], w["tattn.bo"], cfg.heads)
                for f in range(cfg.F):
                    for c in range(C):
                        h[bb * cfg.F + f][c][i][j] += Y[f][c]
    if deep_in is None:
        d0 = conv3x3(h, w["down.w"], w["down.b"], stride=2)
        t = conv3x3(group_norm_silu(d0, w["dres.gn_g"], w["dres.gn_b"], G, cfg.gn_eps), w["dres.w"], w["dres.b"])
        Cd = cfg.C_deep
        deep = [[[[d0[n][c][i][j] + t[n][c][i][j] for j in range(W // 2)] for i in range(H // 2)]
                 for c in range(Cd)] for n in range(N)]
    else:
        deep = deep_in
    cat = [[h[n][c] for c in range(C)] +
           [[[deep[n][c][i // 2][j // 2] for j in range(W)] for i in range(H)] for c in range(cfg.C_deep)]
           for n in range(N)]
    u = conv3x3(group_norm_silu(cat, w["up.gn_g"], w["up.gn_b"], G, cfg.gn_eps), w["up.w"], w["up.b"])
    eps = conv3x3(group_norm_silu(u, w["out.gn_g"], w["out.gn_b"], G, cfg.gn_eps), w["out.w"], w["out.b"])
    return eps, deep


def decoder(cfg, w, z):
    """The latent decoder of the sliced-decoding stage on nested lists z [n][C_lat][H][W], one frame at a time:
    conv_in, residual block, attention block, residual block, then per level residual block, nearest 2x
    upsampling, convolution; GroupNorm, SiLU and a convolution at the end."""
    G = cfg.groups

    def add(a, b):
        return [[[[a[n][c][i][j] + b[n][c][i][j] for j in range(len(a[0][0][0]))] for i in range(len(a[0][0]))]
                 for c in range(len(a[0]))] for n in range(len(a))]

    def res(h, p):
        return add(h, conv3x3(group_norm_silu(h, w[p + ".gn_g"], w[p + ".gn_b"], G, cfg.gn_eps), w[p + ".w"], w[p + ".b"]))

    out = []
    for frame in z:
        h = conv3x3([frame], w["conv_in.w"], w["conv_in.b"])
        h = res(h, "mid.res0")
        C, H, W = len(h[0]), len(h[0][0]), len(h[0][0][0])
        g = group_norm_silu(h, w["mid.attn.gn_g"], w["mid.attn.gn_b"], G, cfg.gn_eps, act=False)
        X = [[g[0][c][i][j] for c in range(C)] for i in range(H) for j in range(W)]
        Y = attn_rows(X, w["mid.attn.wq"], w["mid.attn.wk"], w["mid.attn.wv"], w["mid.attn.wo"], w["mid.attn.bo"], cfg.heads)
        for i in range(H):
            for j in range(W):
                for c in range(C):
                    h[0][c][i][j] += Y[i * W + j][c]
        h = res(h, "mid.res1")
        for l in range(len(cfg.widths) - 1):
            h = res(h, f"up{l}.res")
            H, W = len(h[0][0]), len(h[0][0][0])
            up = [[[[h[0][c][i // 2][j // 2] for j in range(2 * W)] for i in range(2 * H)] for c in range(len(h[0]))]]
            h = conv3x3(up, w[f"up{l}.conv.w"], w[f"up{l}.conv.b"])
        h = conv3x3(group_norm_silu(h, w["out.gn_g"], w["out.gn_b"], G, cfg.gn_eps), w["out.w"], w["out.b"])
        out.append(h[0])
    return out


def dit_blocks(cfg, w, mod, x, i0, i1):
    """Blocks [i0, i1) of the diffusion transformer on nested lists x [T][D] of ONE batch element with that element's
    modulation mod[i] = six lists of D floats; scalar loops throughout. Returns the new x."""
    T, D, H = len(x), cfg.D, cfg.mlp_ratio * cfg.D

    def ln_mod(row, shift, scale):
        mu = sum(row) / D
        var = sum((v - mu) ** 2 for v in row) / D
        r = 1.0 / math.sqrt(var + cfg.ln_eps)
        return [(row[c] - mu) * r * (1.0 + scale[c]) + shift[c] for c in range(D)]

    def lin(row, W, b):
        return [b[o] + sum(W[o][c] * row[c] for c in range(len(row))) for o in range(len(W))]

    x = [list(r) for r in x]
    for i in range(i0, i1):
        m = mod[i]
        h = [ln_mod(r, m[0], m[1]) for r in x]
        qkv = [lin(r, w[f"blk{i}.wqkv"], w[f"blk{i}.bqkv"]) for r in h]
        O = attn_core([r[:D] for r in qkv], [r[D:2 * D] for r in qkv], [r[2 * D:] for r in qkv], cfg.heads)
        for t in range(T):
            y = lin(O[t], w[f"blk{i}.wo"], w[f"blk{i}.bo"])
            for c in range(D):
                x[t][c] += m[2][c] * y[c]
        for t in range(T):
            hrow = ln_mod(x[t], m[3], m[4])
            u = lin(hrow, w[f"blk{i}.w1"], w[f"blk{i}.b1"])
            u = [0.5 * v * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3))) for v in u]
            y = lin(u, w[f"blk{i}.w2"], w[f"blk{i}.b2"])
            for c in range(D):
                x[t][c] += m[5][c] * y[c]
    return x
