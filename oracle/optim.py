"""Parameter updates, written out from their definitions in float64 numpy.  TEST INFRASTRUCTURE ONLY.

sgd:  w - lr (dw + wd w).
adam: Kingma & Ba (2015), Algorithm 1, with the weight decay added to the gradient first.
Pinned in tests/test_oracle_pins.py by closed forms (geometric decay on a quadratic; the first Adam step
has size lr whatever the gradient's scale; a constant gradient keeps every Adam step at lr).
"""
import numpy as np


def sgd(w, dw, lr, wd=0.0):
    w = np.asarray(w, dtype=np.float64)
    return w - lr * (np.asarray(dw, dtype=np.float64) + wd * w)


def adam(w, dw, m, v, t, lr, b1=0.9, b2=0.999, eps=1e-8, wd=0.0):
    """Returns (w, m, v) after step t (t = 1 for the first step)."""
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(dw, dtype=np.float64) + wd * w
    m = b1 * np.asarray(m, dtype=np.float64) + (1.0 - b1) * g
    v = b2 * np.asarray(v, dtype=np.float64) + (1.0 - b2) * g * g
    mhat = m / (1.0 - b1 ** t)
    vhat = v / (1.0 - b2 ** t)
    return w - lr * mhat / (np.sqrt(vhat) + eps), m, v
