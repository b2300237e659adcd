"""Inputs for which a single-precision Hadamard transform misjudges Eq. 5: vectors with a wide
exponent spread (every other element scaled by 2^-10, so that fp32 partial sums round) and
thresholds set to a coefficient's own exact value rounded to float, i.e. a few 1e-8 relative
away from the exact sum, above or below as the rounding falls.  Used by a CPU test (plain fp32
gets them wrong) and a GPU test (the library's bulk and query encodes must get them right)."""

import numpy as np

import synth_inputs as synth

N_VECTORS = 384


def trials(oracle, n_trials=24, seed=77):
    """Yields (bf16 bit patterns [N_VECTORS, 128], thresholds (3 floats), exact sums picked)."""
    rng = np.random.default_rng(seed)
    for _ in range(n_trials):
        x = rng.standard_normal((N_VECTORS, 128), dtype=np.float32)
        x[:, rng.choice(128, 4, replace=False)] *= 8.0
        x[:, 1::2] *= np.float32(2.0 ** -10)
        bits = synth.f32_to_bf16_bits(x)
        xs = synth.bf16_bits_to_f32(bits).astype(np.float64)
        picks = []
        for t in range(3):
            y = oracle.hadamard_transform(xs[17 + 100 * t])
            picks.append(float(y[rng.integers(128)]))
        picks.sort()
        thr = tuple(float(np.float32(v / np.sqrt(128.0))) for v in picks)
        if thr[0] < thr[1] < thr[2]:
            yield bits, thr, picks


def fwht_float32(x):
    """Radix-2 butterflies in float32, every addition rounded (numpy), rows of 128."""
    x = np.asarray(x, dtype=np.float32).copy()
    h = 1
    while h < 128:
        y = x.reshape(-1, 128 // (2 * h), 2, h)
        a, b = y[:, :, 0, :].copy(), y[:, :, 1, :].copy()
        y[:, :, 0, :] = a + b
        y[:, :, 1, :] = a - b
        x = y.reshape(-1, 128)
        h *= 2
    return x
