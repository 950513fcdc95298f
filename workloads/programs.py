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


C3_WEIGHTS = ("Wq", "Wk", "Wv", "Wo", "W1", "W2")
C3_VECTORS = ("bq", "bk", "bv", "bo", "b1", "b2", "g1", "be1", "g2", "be2")


def c3_step(B, x, dy, P, M, V, heads, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, t=1):
    """Pre-LayerNorm transformer encoder layer, forward + backward + Adam, one trace.
    x, dy: [batch, seq, d] bf16 (dy is the upstream gradient of the layer output).
    P: dict of bf16 parameters (C3_WEIGHTS are [in, out] matrices), M / V: dicts of fp32 Adam
    moments with the same keys; all three are updated in place.  Returns (y, dx).
    The 1/sqrt(d_head) factor is folded into the query projection."""
    bsz, seq, d = x.shape
    dh = d // heads
    n = bsz * seq
    scale = 1.0 / (dh ** 0.5)
    x2 = B.reshape(x, (n, d))
    dy2 = B.reshape(dy, (n, d))

    def split(t2):      # [n, d] -> [batch, heads, seq, dh]   (views)
        return B.permute(B.reshape(t2, (bsz, seq, heads, dh)), (0, 2, 1, 3))

    def merge(t4):      # [batch, heads, seq, dh] -> [n, d]
        return B.reshape(B.permute(t4, (0, 2, 1, 3)), (n, d))

    # ---- forward
    ln1, mu1, rs1 = B.layer_norm(x2, P["g1"], P["be1"])
    qs = B.mul(B.add(B.matmul(ln1, P["Wq"]), P["bq"]), scale)
    kk = B.add(B.matmul(ln1, P["Wk"]), P["bk"])
    vv = B.add(B.matmul(ln1, P["Wv"]), P["bv"])
    qh, kh, vh = split(qs), split(kk), split(vv)
    prob = B.softmax(B.matmul(qh, kh, trans_b=True))
    ctx = merge(B.matmul(prob, vh))
    x3 = B.add(x2, B.add(B.matmul(ctx, P["Wo"]), P["bo"]))
    ln2, mu2, rs2 = B.layer_norm(x3, P["g2"], P["be2"])
    u = B.add(B.matmul(ln2, P["W1"]), P["b1"])
    h = B.gelu(u)
    y = B.add(x3, B.add(B.matmul(h, P["W2"]), P["b2"]))

    # ---- backward
    G = {}
    G["W2"] = B.matmul(h, dy2, trans_a=True)
    G["b2"] = B.sum(dy2, axis=0)
    du = B.gelu_grad(B.matmul(dy2, P["W2"], trans_b=True), u)
    G["W1"] = B.matmul(ln2, du, trans_a=True)
    G["b1"] = B.sum(du, axis=0)
    dln2 = B.matmul(du, P["W1"], trans_b=True)
    xhat2 = B.mul(B.sub(x3, B.reshape(mu2, (n, 1))), B.reshape(rs2, (n, 1)))
    G["g2"] = B.sum(B.mul(dln2, xhat2), axis=0)
    G["be2"] = B.sum(dln2, axis=0)
    dx3 = B.add(dy2, B.layer_norm_grad(dln2, x3, P["g2"], mu2, rs2))
    G["Wo"] = B.matmul(ctx, dx3, trans_a=True)
    G["bo"] = B.sum(dx3, axis=0)
    dctx = split(B.matmul(dx3, P["Wo"], trans_b=True))
    dprob = B.matmul(dctx, vh, trans_b=True)
    dvv = merge(B.matmul(prob, dctx, trans_a=True))
    dscore = B.softmax_grad(dprob, prob)
    dqs = merge(B.matmul(dscore, kh))
    dkk = merge(B.matmul(dscore, qh, trans_a=True))
    G["Wq"] = B.mul(B.matmul(ln1, dqs, trans_a=True), scale)
    G["bq"] = B.mul(B.sum(dqs, axis=0), scale)
    G["Wk"] = B.matmul(ln1, dkk, trans_a=True)
    G["bk"] = B.sum(dkk, axis=0)
    G["Wv"] = B.matmul(ln1, dvv, trans_a=True)
    G["bv"] = B.sum(dvv, axis=0)
    dln1 = B.mul(B.matmul(dqs, P["Wq"], trans_b=True), scale)
    dln1 = B.add(B.matmul(dkk, P["Wk"], trans_b=True), dln1)
    dln1 = B.add(B.matmul(dvv, P["Wv"], trans_b=True), dln1)
    xhat1 = B.mul(B.sub(x2, B.reshape(mu1, (n, 1))), B.reshape(rs1, (n, 1)))
    G["g1"] = B.sum(B.mul(dln1, xhat1), axis=0)
    G["be1"] = B.sum(dln1, axis=0)
    dx = B.add(dx3, B.layer_norm_grad(dln1, x2, P["g1"], mu1, rs1))

    # ---- Adam: moments fp32, parameters bf16 (update in fp32, then rounded)
    for name in C3_WEIGHTS + C3_VECTORS:
        g, p, m, v = G[name], P[name], M[name], V[name]
        m_new = B.add(B.mul(m, beta1), g, alpha=1.0 - beta1)
        v_new = B.add(B.mul(v, beta2), B.square(g), alpha=1.0 - beta2)
        mhat = B.div(m_new, 1.0 - beta1 ** t)
        vhat = B.div(v_new, 1.0 - beta2 ** t)
        p_new = B.cast(B.sub(p, B.div(B.mul(mhat, lr), B.add(B.sqrt(vhat), eps))), "bf16")
        B.assign(p, p_new)
        B.assign(m, m_new)
        B.assign(v, v_new)
    return y, dx


def views_program(B, x, y):
    """In-place updates through views (section 4.4 of the paper).  x: [2, 3, 4], y: [6, 4], both
    fp32.  Returns (x, v, w, s): the base, two of its views and a value read from a view after
    other views were updated."""
    v = B.view_permute(x, (1, 2, 0))                  # the view of the paper's figure 3 ...
    B.assign(v, B.add(v, 42.0))                       # ... and its in-place add
    w = B.view_narrow(x, 1, 1, 2)                     # a window along the middle axis
    B.assign(w, B.mul(w, 2.0))                        # the sibling view v must see this
    r = B.view_reshape(x, (6, 4))
    B.assign(r, B.sub(r, y))
    chain = B.view_narrow(B.view_reshape(x, (6, 4)), 0, 2, 3)   # a view of a view
    B.assign(chain, B.neg(chain))
    s = B.add(B.exp(B.mul(v, 0.01)), B.narrow(v, 2, 0, 1))      # reads: a view, and a window of it as a broadcast operand
    B.assign(x, B.mul(x, 0.5))                        # updating the base shows in every view
    return x, v, w, s
