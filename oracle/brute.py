"""Pure-Python-loop twins, for tiny sizes only.  They restate the definitions
with scalars and explicit sums so that a transposed operand, a wrong index or a
dropped term in the array code shows up as a mismatch."""
import math


def mlp_loss(theta, dims, X, y):
    """mean_i l_i computed with scalar loops (no gradient)."""
    rows = len(X)
    L = len(dims) - 1
    total = 0.0
    for i in range(rows):
        h = [float(t) for t in X[i]]
        at = 0
        for l in range(L):
            k, n = dims[l], dims[l + 1]
            z = []
            for j in range(n):
                s = float(theta[at + k * n + j])            # b_l[j]
                for q in range(k):
                    s += h[q] * float(theta[at + q * n + j])  # W_l[q, j]
                z.append(s)
            at += k * n + n
            h = [max(t, 0.0) for t in z] if l < L - 1 else z
        m = max(h)
        lse = m + math.log(sum(math.exp(t - m) for t in h))
        total += lse - h[int(y[i])]
    return total / rows


def mlp_grad_two_layer(theta, dims, X, y):
    """Analytic gradient of mean_i l_i for exactly one hidden layer, element
    by element.  Returns a flat list laid out like theta."""
    d0, d1, d2 = dims
    rows = len(X)
    oW1, ob1 = 0, d0 * d1
    oW2 = ob1 + d1
    ob2 = oW2 + d1 * d2
    g = [0.0] * (ob2 + d2)
    for i in range(rows):
        x = [float(t) for t in X[i]]
        z1 = [float(theta[ob1 + j]) + sum(x[q] * float(theta[oW1 + q * d1 + j]) for q in range(d0))
              for j in range(d1)]
        h1 = [max(t, 0.0) for t in z1]
        z2 = [float(theta[ob2 + c]) + sum(h1[j] * float(theta[oW2 + j * d2 + c]) for j in range(d1))
              for c in range(d2)]
        m = max(z2)
        ex = [math.exp(t - m) for t in z2]
        se = sum(ex)
        dz2 = [(ex[c] / se - (1.0 if c == int(y[i]) else 0.0)) / rows for c in range(d2)]
        for c in range(d2):
            g[ob2 + c] += dz2[c]
            for j in range(d1):
                g[oW2 + j * d2 + c] += h1[j] * dz2[c]
        for j in range(d1):
            if h1[j] > 0.0:
                dz1 = sum(dz2[c] * float(theta[oW2 + j * d2 + c]) for c in range(d2))
                g[ob1 + j] += dz1
                for q in range(d0):
                    g[oW1 + q * d1 + j] += x[q] * dz1
    return g


def momentum_closed_form(p0, g, lr, m, k):
    """p after k steps with a constant gradient g, v0 = 0, no weight decay:
    p_k = p0 - lr * g * sum_{j=1..k} (1 - m^j) / (1 - m)."""
    s = sum((1.0 - m ** j) / (1.0 - m) for j in range(1, k + 1))
    return p0 - lr * g * s


def adam_first_step(p0, g, lr, beta2, eps):
    """Adam's first update from zero moments, element by element: the bias
    corrections cancel beta1 entirely and leave
    p1 = p0 - lr * g / (|g| + eps / sqrt(1 - beta2))."""
    return [float(a) - lr * float(b) / (abs(float(b)) + eps / math.sqrt(1.0 - beta2)) for a, b in zip(p0, g)]


def rmsprop_constant_gradient(p0, g, lr, rho, eps, k):
    """RMSProp after k steps with a constant gradient and a zero accumulator:
    a_j = (1 - rho^j) g^2, so p_k = p0 - lr * g * sum_j 1 / sqrt((1 - rho^j) g^2 + eps)."""
    out = []
    for a, b in zip(p0, g):
        a, b = float(a), float(b)
        out.append(a - lr * b * sum(1.0 / math.sqrt((1.0 - rho ** j) * b * b + eps) for j in range(1, k + 1)))
    return out


def conv3x3_point(X, Wc, i, h, w, o):
    """One output value of the 3x3 convolution with zero padding 1, from its
    definition: the sum over the 3x3 neighbourhood of pixel (h, w), taking
    pixels outside the image as zero.  X: [n][H][W][C_in] nested sequences,
    Wc: [3][3][C_in][C_out]."""
    H, W, C = len(X[0]), len(X[0][0]), len(X[0][0][0])
    s = 0.0
    for dh in (-1, 0, 1):
        for dw in (-1, 0, 1):
            hh, ww = h + dh, w + dw
            if hh < 0 or hh >= H or ww < 0 or ww >= W:
                continue
            for c in range(C):
                s += float(X[i][hh][ww][c]) * float(Wc[dh + 1][dw + 1][c][o])
    return s


def convblock_loss(theta, shape, X, y, eps):
    """The conv + BN block's mean loss with scalar loops only (no gradient).
    X: [n][H][W][C_in]."""
    H, W, cin, cout, classes = shape
    n = len(X)
    oWc, og = 0, 9 * cin * cout
    ob = og + cout
    oWf = ob + cout
    obf = oWf + cout * classes
    Wc = [[[[float(theta[oWc + ((kh * 3 + kw) * cin + c) * cout + o]) for o in range(cout)]
            for c in range(cin)] for kw in range(3)] for kh in range(3)]
    z = [[[[conv3x3_point(X, Wc, i, h, w, o) for o in range(cout)] for w in range(W)]
          for h in range(H)] for i in range(n)]
    cnt = n * H * W
    p = [[0.0] * cout for _ in range(n)]
    for o in range(cout):
        mu = sum(z[i][h][w][o] for i in range(n) for h in range(H) for w in range(W)) / cnt
        var = sum((z[i][h][w][o] - mu) ** 2 for i in range(n) for h in range(H) for w in range(W)) / cnt
        for i in range(n):
            acc = 0.0
            for h in range(H):
                for w in range(W):
                    v = float(theta[og + o]) * (z[i][h][w][o] - mu) / math.sqrt(var + eps) + float(theta[ob + o])
                    acc += max(v, 0.0)
            p[i][o] = acc / (H * W)
    total = 0.0
    for i in range(n):
        logits = [float(theta[obf + k]) + sum(p[i][o] * float(theta[oWf + o * classes + k]) for o in range(cout))
                  for k in range(classes)]
        m = max(logits)
        total += m + math.log(sum(math.exp(t - m) for t in logits)) - logits[int(y[i])]
    return total / n


def bf16_rne(v):
    """One number rounded the way a bf16-input pipeline receives it: to single
    precision first (the precision the surrounding arithmetic runs in; the
    struct module converts with round-to-nearest-even), then to the nearest
    bfloat16, ties to the even neighbour.  Integer arithmetic on the 32-bit
    pattern, one scalar at a time; finite inputs only."""
    import struct
    bits = struct.unpack("<I", struct.pack("<f", float(v)))[0]
    top, low = bits >> 16, bits & 0xFFFF
    if low > 0x8000 or (low == 0x8000 and (top & 1)):
        top += 1                       # a carry into the exponent is the right next value
    return struct.unpack("<f", struct.pack("<I", (top << 16) & 0xFFFFFFFF))[0]


BF16_POINTS = ("x", "w", "h", "dz")


def mlp_loss_grad_bf16_points(theta, dims, X, y, points=BF16_POINTS, rnd=bf16_rne):
    """Loss and gradient of mean_i l_i for any number of layers, scalar loops
    only, with the values a bf16-input contraction is fed rounded by `rnd`:
      "x"   the input rows,
      "w"   every W_l (in the forward product and in the backward product),
      "h"   every hidden activation relu(z_l) as the next layer receives it,
      "dz"  every dZ_l, before any of its three uses (dW_l, db_l, dZ_{l-1}).
    Biases, the softmax, the relu mask (taken from the unrounded z_l) and all
    sums stay in double precision.  `points` names the rounding points that
    are active, so that a test can take one out or put one in the wrong place
    ("b": also round the biases; "late_dz": round dZ_l only where it enters the
    product with W_l^T, not for dW_l and db_l).
    Returns (loss, flat gradient list laid out like theta)."""
    q = lambda v, name: rnd(v) if name in points else float(v)
    L = len(dims) - 1
    rows = len(X)
    offW, offB, at = [], [], 0
    for l in range(L):
        offW.append(at)
        at += dims[l] * dims[l + 1]
        offB.append(at)
        at += dims[l + 1]
    g = [0.0] * at
    Wq = [[[q(theta[offW[l] + a * dims[l + 1] + j], "w") for j in range(dims[l + 1])]
           for a in range(dims[l])] for l in range(L)]
    bq = [[q(theta[offB[l] + j], "b") for j in range(dims[l + 1])] for l in range(L)]
    total = 0.0
    for i in range(rows):
        h = [[q(t, "x") for t in X[i]]]                 # h[l]: what layer l+1's product receives
        pos = []                                         # pos[l][j]: relu(z_{l+1})[j] > 0
        for l in range(L):
            z = [bq[l][j] + sum(h[l][a] * Wq[l][a][j] for a in range(dims[l])) for j in range(dims[l + 1])]
            if l < L - 1:
                pos.append([t > 0.0 for t in z])
                h.append([q(max(t, 0.0), "h") for t in z])
        m = max(z)
        ex = [math.exp(t - m) for t in z]
        se = sum(ex)
        total += m + math.log(se) - z[int(y[i])]
        dz_full = [(ex[c] / se - (1.0 if c == int(y[i]) else 0.0)) / rows for c in range(dims[L])]
        for l in range(L - 1, -1, -1):
            dz_q = [q(t, "dz") for t in dz_full]
            dz_w = dz_full if "late_dz" in points else dz_q    # what dW_l and db_l are built from
            dz_x = [rnd(t) for t in dz_full] if "late_dz" in points else dz_q
            for j in range(dims[l + 1]):
                g[offB[l] + j] += dz_w[j]
                for a in range(dims[l]):
                    g[offW[l] + a * dims[l + 1] + j] += h[l][a] * dz_w[j]
            if l > 0:
                dz_full = [sum(dz_x[j] * Wq[l][a][j] for j in range(dims[l + 1])) if pos[l - 1][a] else 0.0
                           for a in range(dims[l])]
    return total / rows, g
