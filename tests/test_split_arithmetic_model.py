"""Where the split-bf16 tolerances come from: a numpy model of the arithmetic (every iterate and temporary kept as p bf16
planes, every product of Eq. 2 taken over the plane pairs i + j < p, results formed in fp32 and split again), run
against the fp64 oracle.  No GPU and no library code is involved; the model states what the library's rounding points
are, the parity tests check that the library stays inside the same bars."""
import numpy as np
import pytest

from oracle import muon_oracle as orc

A_, B_, C_ = 3.4445, -4.7750, 2.0315


def bf16(x):
    u = np.asarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def split(x, planes):
    rest, out = np.asarray(x, np.float32).copy(), []
    for _ in range(planes):
        h = bf16(rest)
        out.append(h.astype(np.float64))
        rest = (rest - h).astype(np.float32)          # exact: the rounding error of an fp32 value is an fp32 value
    return out


def product(left, right, planes):
    acc = np.zeros((left[0].shape[0], right[0].shape[0]))
    for i in range(planes):
        for j in range(planes - i):
            acc += left[i] @ right[j].T
    return acc


def model(u, planes, steps=5):
    s = 1.0 / np.linalg.norm(u)
    x = split(u, planes)                               # stored un-normalised; s enters in the first two epilogues
    for it in range(steps):
        s2, s1 = (s * s, s) if it == 0 else (1.0, 1.0)
        a = split((s2 * product(x, x, planes)).astype(np.float32), planes)
        b = split((C_ * product(a, a, planes) + B_ * sum(a)).astype(np.float32), planes)
        xt = [p.T for p in x]
        x = split((s1 * (product(b, xt, planes) + A_ * sum(x))).astype(np.float32), planes)
    return sum(x)


@pytest.mark.parametrize("shape", [(96, 160), (128, 256), (256, 512)])
def test_error_level_of_each_plane_count(shape):
    rng = np.random.default_rng(shape[0])
    u = bf16(rng.standard_normal(shape) * 1e-3).astype(np.float64)
    ref = orc.newton_schulz(u, steps=5)
    err = {p: np.linalg.norm(model(u, p) - ref) / np.linalg.norm(ref) for p in (1, 2, 3)}
    assert 3e-3 < err[1] < 2e-2          # plain bf16: the 2e-2 bar
    assert 3e-6 < err[2] < 6e-5          # two planes: below the 1e-4 bar with room for fp32 accumulation order
    assert err[3] < 1e-6                 # three planes: fp32-class; the library's 1e-5 bar is set by its fp32 sums
    assert err[2] < err[1] / 100 and err[3] < err[2] / 30


def test_dropping_a_cross_term_is_visible():
    """The pair list matters: with two planes and only the hi*hi product the result is no better than plain bf16."""
    rng = np.random.default_rng(5)
    u = bf16(rng.standard_normal((96, 160)) * 1e-3).astype(np.float64)
    ref = orc.newton_schulz(u, steps=5)

    def hi_only(left, right, planes):
        return left[0] @ right[0].T

    global product
    full = product
    try:
        product = hi_only
        crippled = np.linalg.norm(model(u, 2) - ref) / np.linalg.norm(ref)
    finally:
        product = full
    assert crippled > 2e-3
