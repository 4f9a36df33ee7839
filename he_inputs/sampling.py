"""Seeded random draws consumed by both the CPU oracle and the HIP path.

Every array is drawn from numpy's PCG64 generator seeded with the workload's seed, so a test
and a benchmark that name the same (config, seed) see the same bits.
"""
import numpy as np


def make_rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def uniform_limbs(rng: np.random.Generator, moduli, N: int, npoly: int = 1) -> np.ndarray:
    """uint64 array [npoly][len(moduli)][N]; limb i uniform in [0, moduli[i])."""
    out = np.empty((npoly, len(moduli), N), dtype=np.uint64)
    for i, m in enumerate(moduli):
        out[:, i, :] = rng.integers(0, int(m), size=(npoly, N), dtype=np.uint64)
    return out


def ternary_secret(rng: np.random.Generator, N: int, hamming: int) -> np.ndarray:
    """int64 array [N] with exactly `hamming` entries in {-1,+1} (equiprobable), the rest 0."""
    s = np.zeros(N, dtype=np.int64)
    pos = rng.choice(N, size=hamming, replace=False)
    s[pos] = rng.integers(0, 2, size=hamming, dtype=np.int64) * 2 - 1
    return s


def gaussian_error(rng: np.random.Generator, N: int, sigma: float = 3.2, n: int = 1) -> np.ndarray:
    """int64 array [n][N]: normal(0, sigma) rounded to nearest, clipped at 6 sigma."""
    e = np.rint(rng.normal(0.0, sigma, size=(n, N)))
    lim = int(np.floor(6 * sigma))
    return np.clip(e, -lim, lim).astype(np.int64)


def conv_tensors(rng: np.random.Generator, c_in: int, c_out: int, H: int, W: int, f: int, w_std: float):
    """Image x ~ U[-1,1]^{c_in x H x W} and filter Wt ~ N(0, w_std^2)^{c_out x c_in x f x f} (float64)."""
    x = rng.uniform(-1.0, 1.0, size=(c_in, H, W))
    wt = rng.normal(0.0, w_std, size=(c_out, c_in, f, f))
    return x, wt
