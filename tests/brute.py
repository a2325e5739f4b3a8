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


def unet_rb(cfg, w, p, x, temb):
    """Residual block with a time embedding on nested lists x [N][Cin][H][W], temb [B][temb_dim] (frame n belongs to
    batch element n // (N / B)): two GroupNorm-SiLU-conv3x3 stages, the projected SiLU(temb) added per channel
    between them, a 1x1 shortcut when the block has one."""
    N, Cin, H, W = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0])
    Cout = len(w[p + ".conv1.b"])
    per = N // len(temb)
    h = conv3x3(group_norm_silu(x, w[p + ".gn1_g"], w[p + ".gn1_b"], cfg.groups, cfg.gn_eps), w[p + ".conv1.w"], w[p + ".conv1.b"])
    for n in range(N):
        tb = temb[n // per]
        st = [v / (1.0 + math.exp(-v)) for v in tb]
        for o in range(Cout):
            add = w[p + ".temb.b"][o] + sum(w[p + ".temb.w"][o][k] * st[k] for k in range(len(st)))
            for i in range(H):
                for j in range(W):
                    h[n][o][i][j] += add
    y = conv3x3(group_norm_silu(h, w[p + ".gn2_g"], w[p + ".gn2_b"], cfg.groups, cfg.gn_eps), w[p + ".conv2.w"], w[p + ".conv2.b"])
    for n in range(N):
        for o in range(Cout):
            for i in range(H):
                for j in range(W):
                    if (p + ".short.w") in w:
                        sc = w[p + ".short.b"][o] + sum(w[p + ".short.w"][o][c] * x[n][c][i][j] for c in range(Cin))
                    else:
                        sc = x[n][o][i][j]
                    y[n][o][i][j] += sc
    return y


def unet_tf_rows(cfg, w, p, Z, ctx=None, pe=None):
    """The token part of a transformer block on ONE sequence Z (rows of C floats, already projected in): self-attention
    on LayerNorm'ed rows (+ pe[row] when given), cross-attention against the rows `ctx` when given, GEGLU feed-forward;
    each with its residual. Returns the new rows."""
    C = len(Z[0])
    heads = C // cfg.head_dim

    def ln(row, q):
        mu = sum(row) / C
        var = sum((v - mu) ** 2 for v in row) / C
        r = 1.0 / math.sqrt(var + cfg.ln_eps)
        return [(row[c] - mu) * r * w[f"{p}.{q}_g"][c] + w[f"{p}.{q}_b"][c] for c in range(C)]

    def lin(row, W, b=None):
        return [(b[o] if b is not None else 0.0) + sum(W[o][c] * row[c] for c in range(len(row))) for o in range(len(W))]

    def attend(Qin, KVin, a):
        O = attn_core([lin(r, w[f"{p}.{a}.wq"]) for r in Qin], [lin(r, w[f"{p}.{a}.wk"]) for r in KVin],
                      [lin(r, w[f"{p}.{a}.wv"]) for r in KVin], heads)
        return [lin(r, w[f"{p}.{a}.wo"], w[f"{p}.{a}.bo"]) for r in O]

    Z = [list(r) for r in Z]
    A = [ln(r, "ln1") for r in Z]
    if pe is not None:
        A = [[A[t][c] + pe[t][c] for c in range(C)] for t in range(len(A))]
    Y = attend(A, A, "attn1")
    Z = [[Z[t][c] + Y[t][c] for c in range(C)] for t in range(len(Z))]
    if ctx is not None:
        Y = attend([ln(r, "ln2") for r in Z], ctx, "attn2")
        Z = [[Z[t][c] + Y[t][c] for c in range(C)] for t in range(len(Z))]
    for t in range(len(Z)):
        u = lin(ln(Z[t], "ln3"), w[p + ".ff1.w"], w[p + ".ff1.b"])
        half = len(u) // 2
        gl = [u[k] * (0.5 * u[half + k] * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (u[half + k] + 0.044715 * u[half + k] ** 3))))
              for k in range(half)]
        y = lin(gl, w[p + ".ff2.w"], w[p + ".ff2.b"])
        for c in range(C):
            Z[t][c] += y[c]
    return Z


def frame_pe(F, C):
    """pe[f][2i] = sin(f / 10000^(2i/C)), pe[f][2i+1] = cos(f / 10000^(2i/C))."""
    return [[(math.sin if c % 2 == 0 else math.cos)(f / 10000.0 ** ((c - c % 2) / C)) for c in range(C)] for f in range(F)]


def unet_tf(cfg, w, p, x, ctx=None, temporal=False):
    """A transformer block on nested lists x [N][C][H][W]: GroupNorm, projection in, the token part over the positions
    of each frame (spatial; ctx [B][L][ctx_dim]) or over the F frames of each position with the frame positional encoding
    (temporal), projection out, residual."""
    N, C, H, W = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0])
    g = group_norm_silu(x, w[p + ".gn_g"], w[p + ".gn_b"], cfg.groups, cfg.gn_eps, act=False)

    def lin(row, W_, b):
        return [b[o] + sum(W_[o][c] * row[c] for c in range(len(row))) for o in range(len(W_))]

    y = [[[[x[n][c][i][j] for j in range(W)] for i in range(H)] for c in range(C)] for n in range(N)]
    if not temporal:
        per = N // len(ctx)
        for n in range(N):
            Z = [lin([g[n][c][i][j] for c in range(C)], w[p + ".pin.w"], w[p + ".pin.b"]) for i in range(H) for j in range(W)]
            Z = unet_tf_rows(cfg, w, p, Z, ctx=ctx[n // per])
            for i in range(H):
                for j in range(W):
                    o = lin(Z[i * W + j], w[p + ".pout.w"], w[p + ".pout.b"])
                    for c in range(C):
                        y[n][c][i][j] += o[c]
    else:
        F = N // cfg.B
        pe = frame_pe(F, C)
        for b in range(cfg.B):
            for i in range(H):
                for j in range(W):
                    Z = [lin([g[b * F + f][c][i][j] for c in range(C)], w[p + ".pin.w"], w[p + ".pin.b"]) for f in range(F)]
                    Z = unet_tf_rows(cfg, w, p, Z, pe=pe)
                    for f in range(F):
                        o = lin(Z[f], w[p + ".pout.w"], w[p + ".pout.b"])
                        for c in range(C):
                            y[b * F + f][c][i][j] += o[c]
    return y
