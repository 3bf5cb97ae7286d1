"""Host-side check of the arithmetic shortcut the activation kernels take: the code rne(x / s) may be read off
t = x * (1 / s) whenever t is at least 5e-5 away from a half-integer.  Exercised in IEEE single precision with numpy on
random rows and on values placed next to rounding boundaries; the kernels themselves are compared with the oracle,
bit for bit, in the GPU tests."""
import numpy as np

import synth_inputs as S

F = np.float32


def _check(x, s):
    x = x.astype(F)
    r = F(1.0) / s
    t = x * r
    q_fast = np.rint(t)
    safe = np.abs(t - q_fast) <= F(0.49995)
    q_true = np.rint(x / s)
    assert np.array_equal(q_fast[safe], q_true[safe])
    return int((~safe).sum()), x.size


def test_reciprocal_codes_equal_quotient_codes_where_claimed():
    unsafe = total = 0
    for seed in range(6):
        x = S.activations_outlier(64, 4096, seed=900 + seed).astype(np.float16)
        for row in x:
            amax = F(np.abs(row.astype(F)).max())
            u, n = _check(row, amax / F(127.0))
            unsafe += u
            total += n
    assert unsafe < 1e-3 * total        # the fallback is rare


def test_values_next_to_rounding_boundaries():
    rng = np.random.default_rng(5)
    for _ in range(200):
        amax = F(np.float16(rng.uniform(0.5, 300.0)))
        s = amax / F(127.0)
        k = rng.integers(-127, 127, size=512)
        # fp16 values as close as fp16 allows to (k + 1/2) s, on both sides
        x = ((k + 0.5) * float(s)).astype(np.float16)
        near = np.concatenate([x, np.nextafter(x, np.float16(np.inf)), np.nextafter(x, np.float16(-np.inf))])
        near = near[np.abs(near.astype(F)) <= amax]
        _check(near, s)
