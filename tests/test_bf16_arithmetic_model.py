"""A numpy model of the bf16 Newton-Schulz arithmetic (X, A, B stored in bf16, products and epilogues exact until the one
rounding) against the fp64 oracle, for the formulations of one iteration of Eq. 2 that were considered:

  explicit   B = b A + c A A,                X' = a X + B X        (the a X term an fp32 addend of the last product)
  folded     B' = b A + c A A + a I,         X' = B' X             (what the library does for m >= 64)
  square     A~ = A + b/(2c) I,  B' = c A~ A~ + (a - b^2/(4c)) I   (no addend in the polynomial either)
  one-sided  B' = c A (A + b/c I) + a I                            (the same, shifting one operand only)

The test pins the two facts the design rests on: folding the identity costs no accuracy, and removing the polynomial's
addend by shifting diagonals does.  No GPU and no library code is involved."""
import numpy as np

from oracle import muon_oracle as orc

A_, B_, C_ = 3.4445, -4.7750, 2.0315


def bf16(x):
    u = np.asarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def model(u, mode, steps=5):
    m = u.shape[0]
    s = 1.0 / np.linalg.norm(u)
    x, eye = bf16(u), np.eye(m)
    for it in range(steps):
        s2, s1 = (s * s, s) if it == 0 else (1.0, 1.0)
        g = s2 * (x @ x.T)
        if mode == "explicit":
            a = bf16(g)
            x = bf16(s1 * (A_ * x + bf16(C_ * (a @ a) + B_ * a) @ x))
        elif mode == "folded":
            a = bf16(g)
            x = bf16(s1 * (bf16(C_ * (a @ a) + B_ * a + A_ * eye) @ x))
        elif mode == "square":
            a = bf16(g + B_ / (2 * C_) * eye)
            x = bf16(s1 * (bf16(C_ * (a @ a) + (A_ - B_ * B_ / (4 * C_)) * eye) @ x))
        else:
            a, r = bf16(g), bf16(g + B_ / C_ * eye)
            x = bf16(s1 * (bf16(C_ * (a @ r) + A_ * eye) @ x))
    return x


def test_folding_is_free_and_diagonal_shifts_are_not():
    modes = ("explicit", "folded", "square", "one-sided")
    err = {k: [] for k in modes}
    for shape in ((96, 160), (192, 320), (256, 256)):
        for seed in range(4):
            u = bf16(np.random.default_rng(seed).standard_normal(shape) * 1e-3)
            ref = orc.newton_schulz(u, steps=5)
            for k in modes:
                err[k].append(np.linalg.norm(model(u, k) - ref) / np.linalg.norm(ref))
    mean = {k: float(np.mean(v)) for k, v in err.items()}
    print(mean)
    assert max(err["explicit"]) < 2e-2 and max(err["folded"]) < 2e-2          # both inside the bf16 bar
    assert mean["folded"] <= 1.02 * mean["explicit"]
    assert mean["square"] > 1.05 * mean["folded"]
    assert mean["one-sided"] > 1.25 * mean["folded"]
