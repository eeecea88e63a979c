"""Pure-Python (lists + math, no numpy) brute force for toy layers -- TEST INFRASTRUCTURE ONLY.

An independent second statement of the same definitions as ``clada_oracle.c``,
usable only on tiny shapes (d, d_ff, T <= ~16).  The C oracle is pinned against
this; the two share no code.
"""
import math


def silu(g):
    return g / (1.0 + math.exp(-g))


def gelu_tanh(g):
    """Tanh form of GELU, the gate activation of the Gemma model in the paper's experiments."""
    return 0.5 * g * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (g + 0.044715 * g ** 3)))


def dot(u, v):
    s = 0.0
    for a, b in zip(u, v):
        s += a * b
    return s


def neuron_terms(w_gate, w_up, x, sigma=silu):
    """(a_j, u_j, h_j) of every neuron for one token x."""
    out = []
    for wg, wu in zip(w_gate, w_up):
        a = sigma(dot(wg, x))
        u = dot(wu, x)
        out.append((a, u, a * u))
    return out


def ffn_for_subset(w_gate, w_up, w_down, x, subset, sigma=silu):
    """y = sum_{j in subset} h_j * W_down[j,:], j ascending."""
    d = len(x)
    terms = neuron_terms(w_gate, w_up, x, sigma)
    y = [0.0] * d
    for j in sorted(subset):
        h = terms[j][2]
        for i in range(d):
            y[i] += h * w_down[j][i]
    return y


def kept_set(w_gate, x, tau, sigma=silu):
    """Neurons with |sigma(gate)| >= tau (cut iff strictly below)."""
    return [j for j, wg in enumerate(w_gate) if abs(sigma(dot(wg, x))) >= tau]


def all_subset_outputs(w_gate, w_up, w_down, x):
    """Outputs of all 2^F masks of a toy layer, keyed by the mask's bit pattern."""
    F = len(w_gate)
    return {bits: ffn_for_subset(w_gate, w_up, w_down, x,
                                 [j for j in range(F) if bits >> j & 1])
            for bits in range(1 << F)}


def neuron_magnitude(w_gate, w_up, w_down, X, j):
    """A_j of the neuron-activation equation by its literal reading: the
    Frobenius norm of the rank-one T x d matrix h_{:,j} W_down[j,:]."""
    s = 0.0
    for x in X:
        h = silu(dot(w_gate[j], x)) * dot(w_up[j], x)
        for wd in w_down[j]:
            s += (h * wd) ** 2
    return math.sqrt(s)


def softmax_signals(z, tok):
    """(surprisal, entropy) of one logits row by direct normalisation."""
    m = max(z)
    e = [math.exp(v - m) for v in z]
    Z = sum(e)
    p = [v / Z for v in e]
    H = -sum(q * math.log(q) for q in p if q > 0.0)
    return -math.log(p[tok]), H


def cett_token(w_gate, w_up, w_down, x, eps):
    """CETT of one token: norm of the summed contributions of the neurons with |a| < eps over the
    norm of the dense output (0 when the dense output is zero)."""
    terms = neuron_terms(w_gate, w_up, x)
    cut = [j for j, (a, _, _) in enumerate(terms) if abs(a) < eps]
    yc = ffn_for_subset(w_gate, w_up, w_down, x, cut)
    yf = ffn_for_subset(w_gate, w_up, w_down, x, range(len(w_gate)))
    nf = math.sqrt(sum(v * v for v in yf))
    return math.sqrt(sum(v * v for v in yc)) / nf if nf > 0.0 else 0.0


def cett_argmax(w_gate, w_up, w_down, X, bound):
    """Largest feasible cut threshold by trying every candidate: each pooled magnitude, and one
    value above them all (returned as inf when even that is feasible); None if none is."""
    mags = sorted({abs(a) for x in X for (a, _, _) in neuron_terms(w_gate, w_up, x)})
    best = None
    for eps in mags + [2.0 * mags[-1] + 1.0]:
        m = sum(cett_token(w_gate, w_up, w_down, x, eps) for x in X) / len(X)
        if m <= bound:
            best = eps
    if best is not None and best > mags[-1]:
        return math.inf
    return best
