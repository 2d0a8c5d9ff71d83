"""Oracle of the strategy search's similarity test (Sec. 3.1.2, Algorithm 1 "Avg_Cos_Sim").

Test infrastructure only.  hidden_shared, hidden_original: [S, N] arrays (float32, or uint16
holding bf16 bits), one flattened last-layer hidden state per calibration sentence.
  mode 0: the representations are averaged over the sentences, then one cosine is taken
          (the text of Sec. 3.1.2);
  mode 1: one cosine per sentence, averaged (the procedure's name).
A zero vector is given a cosine of 0.  Everything in float64.
"""
import numpy as np


def _f64(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _cos(x, y):
    nx, ny = np.sqrt((x * x).sum()), np.sqrt((y * y).sum())
    return float((x * y).sum() / (nx * ny)) if nx > 0 and ny > 0 else 0.0


def avg_cos_sim(hidden_shared, hidden_original, mode=0):
    a, b = _f64(hidden_shared), _f64(hidden_original)
    assert a.shape == b.shape and a.ndim == 2
    if mode == 0:
        return _cos(a.mean(axis=0), b.mean(axis=0))
    return float(np.mean([_cos(a[s], b[s]) for s in range(a.shape[0])]))
