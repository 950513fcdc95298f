"""The three small programs whose IR the paper prints (figures 1-3), written
against the abstract tensor API so that both the library's recorder and the
structural oracle can be asked to reproduce the printed listings.

The scaled second operand of a framework `add` is spelled out as
mul(other, expand(alpha)) exactly as section 4.1 describes for figure 1.
"""


def fig1(B, mk):
    """x * y + z on f32[2,4].  mk(shape) makes a device tensor."""
    x, y, z = mk((2, 4)), mk((2, 4)), mk((2, 4))
    prod = B.mul(x, y)
    scaled = B.mul(z, B.expand(B.scalar(1.0), (2, 4)))
    out = B.add(prod, scaled)
    return [out], [x, y, z]


def fig2(B, mk):
    """s = zeros(2,4); twice: s = s + x."""
    x = mk((2, 4))
    s = B.expand(B.scalar(0.0), (2, 4))
    for _ in range(2):
        s = B.add(s, B.mul(x, B.expand(B.scalar(1.0), (2, 4))))
    return [s], [x]


def fig3(B, mk):
    """x of shape (2,3,4); v = x.permute(1,2,0).add_(42): v is a view of x, and the in-place add
    on it makes the recorder write the forward sequence (the view's new value) and the backward
    sequence (x rebuilt through the inverse permutation) by itself.  Only x stays alive."""
    x = mk((2, 3, 4))
    v = B.view_permute(x, (1, 2, 0))
    other = B.mul(B.scalar(42, dtype="s64"), B.scalar(1, dtype="s64"))
    B.assign(v, B.add(v, other))
    del v, other
    return [x], []
