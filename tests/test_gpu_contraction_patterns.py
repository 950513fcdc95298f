"""Random contraction patterns on the GPU against the fp64 oracle: every transpose flag, ragged and
aligned sizes, k from 3 to 5000 (split or not), epilogues with row / full / scalar operands,
attention-like head splits and merges through reshape + permute (operand strides and the sealed
output layout), batched products with a shared weight, weight-gradient shapes with an optimiser-like
epilogue and the column sum next to them; fp32 and bf16."""
import numpy as np
import pytest

from oracle.numeric import Eager, round_to_bf16


def contraction_trace(seed, dt):
    def build(B, mk):
        rg = np.random.Generator(np.random.PCG64(seed))
        ch = lambda xs: xs[int(rg.integers(0, len(xs)))]
        out = []
        kind = int(rg.integers(0, 4))
        if kind == 0:      # plain 2-D with flags and an epilogue
            m, n, k = ch([1, 7, 64, 100, 128, 257]), ch([8, 10, 64, 128, 200, 520]), ch([3, 16, 64, 100, 1024, 4100])
            ta, tb = bool(rg.integers(0, 2)), bool(rg.integers(0, 2))
            a = mk((k, m) if ta else (m, k)); b = mk((n, k) if tb else (k, n))
            y = B.mul(B.matmul(a, b, trans_a=ta, trans_b=tb), 1.0 / k ** 0.5)
            e = int(rg.integers(0, 5))
            if e == 1: y = B.add(y, mk((n,)))
            elif e == 2: y = B.gelu(B.add(y, mk((n,))))
            elif e == 3: y = B.add(B.relu(y), mk((m, n)))
            elif e == 4: y = B.sub(mk((m, n)), B.mul(y, 0.5))
            out.append(y)
            if rg.integers(0, 2): out.append(B.sum(y, axis=0))
        elif kind == 1:    # head split: [b, s, h*d] -> [b, h, s, d], scores, softmax, context, merge
            b_, s, h, d = ch([1, 2, 3]), ch([8, 24, 64, 130]), ch([1, 2, 4]), ch([8, 16, 64])
            q, k_, v = (mk((b_, s, h * d)) for _ in range(3))
            split = lambda t: B.permute(B.reshape(t, (b_, s, h, d)), (0, 2, 1, 3))
            qh, kh, vh = split(q), split(k_), split(v)
            sc = B.mul(B.matmul(qh, kh, trans_b=True), 1.0 / d ** 0.5)
            p = B.softmax(sc)
            c = B.matmul(p, vh)
            merged = B.reshape(B.permute(c, (0, 2, 1, 3)), (b_, s, h * d))
            out += [merged, p] if rg.integers(0, 2) else [merged]
            if rg.integers(0, 2):   # the backward-like products
                dc = split(mk((b_, s, h * d)))
                out.append(B.matmul(p, dc, trans_a=True))
                out.append(B.matmul(dc, vh, trans_b=True))
        elif kind == 2:    # batched with a broadcast weight, rank 3
            b_, m, n, k = ch([2, 5]), ch([16, 33, 128]), ch([8, 64, 136]), ch([16, 64, 200])
            a = mk((b_, m, k)); w = mk((k, n))
            y = B.matmul(B.reshape(a, (b_ * m, k)), w)
            y = B.add(y, mk((n,)))
            out.append(B.reshape(y, (b_, m, n)))
            a2 = mk((b_, k, m)); c2 = mk((b_, k, n))
            out.append(B.matmul(a2, c2, trans_a=True))
        else:              # weight-gradient shape (long k: split) with an optimiser-like epilogue
            m, n, k = ch([64, 128, 256]), ch([64, 128, 520]), ch([2048, 4096, 5000])
            x = mk((k, m)); dy = mk((k, n)); w = mk((m, n)); mom = mk((m, n), "f32")
            g = B.mul(B.matmul(x, dy, trans_a=True), 1.0 / k)
            mom2 = B.add(B.mul(mom, 0.9), B.cast(g, "f32"), alpha=0.1)
            out += [mom2, B.sub(w, B.cast(B.mul(mom2, 0.01), dt))]
            out.append(B.sum(dy, axis=0))
        return out
    return build



@pytest.fixture(scope="module")
def ctx():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2102_13267_amd import Context
    c = Context(device=0, workspace_bytes=2 << 30)
    yield c
    c.close()


@pytest.mark.gpu
@pytest.mark.parametrize("dt,first", [("f32", 0), ("f32", 40), ("bf16", 0), ("bf16", 40)])
def test_random_contraction_patterns(ctx, dt, first):
    """Bar: 2e-5 (fp32: products of up to 5000 terms) / 2e-2 (bf16) of max|ref|, plus twenty times
    the distance of the oracle in working precision from the fp64 oracle."""
    tol0 = 2e-5 if dt == "f32" else 2e-2
    for seed in range(first, first + 40):
        g = np.random.Generator(np.random.PCG64(90000 + seed))
        data = []

        def mk(shape, d=None, donatable=False):
            d = d or dt
            a = (g.standard_normal(shape) * 0.5).astype(np.float32)
            data.append((round_to_bf16(a) if d == "bf16" else a, d))
            return ctx.tensor(data[-1][0].copy(), dtype=d)
        got = contraction_trace(seed, dt)(ctx, mk)
        ctx.barrier()
        refs = []
        for E in (Eager(), Eager("f64")):
            it = iter(data)

            def mk_e(shape, d=None, donatable=False, E=E, it=it):
                a, dd = next(it)
                return E.tensor(a.copy(), dtype=dd)
            refs.append([np.asarray(E.fetch(t), np.float64) for t in contraction_trace(seed, dt)(E, mk_e)])
        for k, (a, rb, rc) in enumerate(zip(got, *refs)):
            ga = np.asarray(ctx.fetch(a), np.float64)
            assert ga.shape == rc.shape, (seed, k)
            scale = max(float(np.max(np.abs(rc))), 1e-2)
            cond = float(np.max(np.abs(rb - rc))) / scale
            err = float(np.max(np.abs(ga - rc))) / scale
            assert np.isfinite(ga).all() and err <= tol0 + 20 * cond, (seed, k, a.shape, err, cond)
        del got
