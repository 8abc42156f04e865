"""How far two CORRECT bf16 implementations of one training step may differ, measured on the oracle alone.

The backward pass takes integer decisions on stored activations: the ReLU mask (y > 0) and the position of a
pooling window's maximum.  An implementation that accumulates in float32 in another order than a second one
produces pre-rounding values that differ by a few parts in 1e6; after rounding to bfloat16 a small share of the
stored activations differs by one unit in the last place, the next layer's pre-activations move by about 2^-9 of
their size, and the decisions of elements that close to zero (or to their window neighbour) flip.  A flipped
decision moves a whole gradient element, so per-tensor infinity-norm errors of earlier layers' gradients grow far
beyond any arithmetic tolerance, on either side.

`order_noise_store` models exactly that and nothing else: every value is multiplied by (1 + r), r uniform in
[-REL, REL], before it is rounded to bfloat16 and stored -- the arithmetic stays fp64.  Comparing the oracle run
with this store against the oracle run with plain rounding gives the decision-flip noise floor of a workload:
the distance between two valid results.  Used by the CPU test of that floor, by the script that writes the
full-size expected values (tests/golden/make_full_step.py) and by the GPU tests' bound on end-to-end gradients.
"""
import numpy as np

from oracle import lpm_oracle as orc

# float32 accumulation of K ~ 1e3..1e4 products in a different order: relative difference of a few eps_f32 * sqrt(K)
REL = 4e-6


def order_noise_store(seed):
    r = np.random.default_rng(seed)

    def store(a):
        a = np.asarray(a, dtype=np.float64)
        return orc.round_bf16(a * (1.0 + r.uniform(-REL, REL, size=a.shape)))

    return store


def inf_err(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def l2_err(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm((got - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-30))


def decision_disagreements(layers, first, last, stash_a, stash_b):
    """Counts, over the layers [first, last), the stored-activation decisions on which two forward states differ:
    ReLU masks (y > 0) of conv/FC layers with ReLU, and first-maximum positions of 2x2 pooling windows.
    Returns (relu_flips, relu_total, pool_flips, pool_total)."""
    rf = rt = pf = pt = 0
    for i in range(first, last):
        l = layers[i]
        if l["kind"] in ("conv", "fc") and l["relu"] and i in stash_a and i in stash_b:
            a, b = np.asarray(stash_a[i]) > 0, np.asarray(stash_b[i]) > 0
            rf += int((a != b).sum()); rt += a.size
        if l["kind"] == "maxpool2" and l["src"] in stash_a and l["src"] in stash_b:
            pa, pb = _argmax2x2(stash_a[l["src"]]), _argmax2x2(stash_b[l["src"]])
            pf += int((pa != pb).sum()); pt += pa.size
    return rf, rt, pf, pt


def _argmax2x2(x):
    """Index 0..3 (row-major in the window) of the first maximum of every 2x2 window of [N][C][H][W]."""
    x = np.asarray(x, dtype=np.float64)
    n, c, h, w = x.shape
    win = x.reshape(n, c, h // 2, 2, w // 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(n, c, h // 2, w // 2, 4)
    return win.argmax(axis=-1)          # numpy returns the first maximum


def window_sums(dx):
    """Sum of every 2x2 window of a pooling layer's input gradient [N][C][H][W]: equal to the pooling output's
    gradient whichever window element received it."""
    dx = np.asarray(dx, dtype=np.float64)
    n, c, h, w = dx.shape
    return dx.reshape(n, c, h // 2, 2, w // 2, 2).sum(axis=(3, 5))
