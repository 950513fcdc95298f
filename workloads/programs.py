"""The user programs of the benchmark configurations, written once against an
abstract tensor API ``B`` (the lazy HIP front end, the eager CPU oracle and the
structural tracer all provide it).  These are inputs to the method -- the
sequence of tensor ops a user's step function issues -- not part of it.
"""
from __future__ import annotations


def c1_trace(B, x, y, bias):
    """out = s / max|s|, s = sum_j z, z = tanh(x*y + bias) * exp(-x^2) + 0.5*y.
    Twelve ops: one broadcast (bias), two reductions."""
    t = B.tanh(B.add(B.mul(x, y), bias))
    e = B.exp(B.neg(B.square(x)))
    z = B.add(B.mul(t, e), y, alpha=0.5)
    s = B.sum(z, axis=1)
    return B.div(s, B.amax(B.abs(s)))


def adam_update(B, p, g, m, v, lr, beta1, beta2, eps, t, clip=None):
    """One Adam step (Kingma & Ba) on (p, m, v), all updated in place; the
    gradient is first scaled by `clip` when given."""
    if clip is not None:
        g = B.mul(g, clip)
    m_new = B.add(B.mul(m, beta1), g, alpha=1.0 - beta1)
    v_new = B.add(B.mul(v, beta2), B.square(g), alpha=1.0 - beta2)
    mhat = B.div(m_new, 1.0 - beta1 ** t)
    vhat = B.div(v_new, 1.0 - beta2 ** t)
    p_new = B.sub(p, B.div(B.mul(mhat, lr), B.add(B.sqrt(vhat), eps)))
    B.assign(p, p_new)
    B.assign(m, m_new)
    B.assign(v, v_new)


def c4_step(B, p, g, m, v, lr, beta1, beta2, eps, t, max_norm):
    """Gradient-norm clipping followed by Adam over one flat parameter vector:
    c = min(1, max_norm / (||g||_2 + 1e-6)), g <- c g, then Adam."""
    gnorm = B.sqrt(B.sum(B.square(g)))
    clip = B.minimum(1.0, B.div(max_norm, B.add(gnorm, 1e-6)))
    adam_update(B, p, g, m, v, lr, beta1, beta2, eps, t, clip=clip)


def c2_step(B, X, labels, params, lr):
    """One SGD step of a ReLU MLP with softmax cross-entropy.
    params = [W1, b1, W2, b2, ...] (updated in place).  Returns the mean loss."""
    n_layers = len(params) // 2
    acts = [X]
    h = X
    for i in range(n_layers):
        W, b = params[2 * i], params[2 * i + 1]
        z = B.add(B.matmul(h, W), b)
        h = B.relu(z) if i < n_layers - 1 else z
        acts.append(h)
    logits = acts[-1]
    loss = B.mean(B.xent(logits, labels))
    batch = X.shape[0]
    d = B.xent_grad(logits, labels, 1.0 / batch)
    updates = []
    for i in reversed(range(n_layers)):
        W, b = params[2 * i], params[2 * i + 1]
        dW = B.matmul(acts[i], d, trans_a=True)
        db = B.sum(d, axis=0)
        if i > 0:
            d = B.relu_grad(B.matmul(d, W, trans_b=True), acts[i])
        updates.append((W, B.sub(W, B.mul(dW, lr))))
        updates.append((b, B.sub(b, B.mul(db, lr))))
    for dst, src in updates:
        B.assign(dst, src)
    return loss


def c5_forward(B, X, W, b, Wr, br, depth):
    """Four GELU layers, then `depth` residual GELU blocks; returns sum(h) as a
    checksum.  `depth` is a host integer: the loop unrolls into the trace."""
    h = X
    for Wi, bi in zip(W, b):
        h = B.gelu(B.add(B.matmul(h, Wi), bi))
    for j in range(depth):
        h = B.add(h, B.gelu(B.add(B.matmul(h, Wr[j]), br[j])))
    return B.sum(h), h
