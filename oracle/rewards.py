"""Synthetic leaf rewards for the oracle (test infrastructure).

Alg. 1 evaluates reward models on the leaves; those models are not available,
so the workloads define stand-ins on the final latent z_T (not from the paper):

  linear       r = <w, z_T> / sqrt(D)
  tanh         r = tanh(<w, z_T> / sqrt(D))
  video        m[f, c] = mean over (h, w) of channel c, frame f;
               r = sum_{f,c} w[f, c] m[f, c] / sqrt(F C)
                   - lam / (F - 1) * sum_f || m[f+1] - m[f] ||^2

PARITY UNPINNED against the paper (these are workload definitions); the tests
pin them against hand values only.
"""
import numpy as np


def reward_linear(z_leaves, w, use_tanh=False):
    z = np.asarray(z_leaves, np.float64)
    r = z @ np.asarray(w, np.float64) / np.sqrt(z.shape[1])
    return np.tanh(r) if use_tanh else r


def reward_video(z_leaves, w, latent_c, latent_t, latent_h, latent_w, lam=1.0):
    """z_leaves [n, D] with the latent stored [C, F, H, W]; w [F, C]."""
    z = np.asarray(z_leaves, np.float64)
    n = z.shape[0]
    m = z.reshape(n, latent_c, latent_t, latent_h * latent_w).mean(axis=3)   # [n, C, F]
    m = m.transpose(0, 2, 1)                                                # [n, F, C]
    lin = (m * np.asarray(w, np.float64)[None]).sum(axis=(1, 2)) / np.sqrt(latent_t * latent_c)
    if latent_t > 1:
        pen = ((m[:, 1:] - m[:, :-1]) ** 2).sum(axis=(1, 2)) / (latent_t - 1)
    else:
        pen = np.zeros(n)
    return lin - lam * pen
