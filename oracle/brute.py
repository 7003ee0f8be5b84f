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
