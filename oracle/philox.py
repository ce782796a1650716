"""Counter-based Gaussian sketch for step 1 of Algorithm 1 (oracle side).

The paper only says the sketching matrix S (n x s, s = k + p) is Gaussian and
drawn on the device by a custom generator (Algorithm 1 step 1; step-1 note in
the method section).  The stream itself is this build's choice: Philox4x32
with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11) followed by Box-Muller.

Mapping (the HIP kernel implements the same one independently):
  key      = (seed & 0xffffffff, seed >> 32)
  counter  = (g & 0xffffffff, g >> 32, stream, 0),  g = group index
  element  e = i * l + j   (row i of Omega, column j)
  fp32: g = e >> 2, lane = e & 3.  x0..x3 -> u_t = ((x_t >> 8) + 0.5) * 2^-24.
        lanes 0,1 = Box-Muller(u0, u1); lanes 2,3 = Box-Muller(u2, u3).
  fp64: g = e >> 1, lane = e & 1.  u0 = (((x0 << 32 | x1) >> 12) + 0.5) * 2^-52,
        u1 likewise from (x2, x3); lanes 0,1 = Box-Muller(u0, u1).
  Box-Muller(u, v): r = sqrt(-2 ln u); (r cos(2 pi v), r sin(2 pi v)),
        with 2 pi v formed as fl(2 pi) * v in one multiplication.
Both uniforms are exact fp64 numbers strictly inside (0, 1).  All transcendental
work is done in fp64 and rounded once to the target dtype.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint64(0x9E3779B9)
_W1 = np.uint64(0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)

TWO_PI = 2.0 * np.pi


def philox4x32_10(counter, key):
    """Philox4x32-10 block function.

    counter: integer array (..., 4), each entry < 2^32; key: two integers < 2^32.
    Returns a uint32 array of the same shape.
    """
    counter = np.asarray(counter)
    c0, c1, c2, c3 = (counter[..., i].astype(np.uint64) for i in range(4))
    k0 = np.uint64(int(key[0]) & 0xFFFFFFFF)
    k1 = np.uint64(int(key[1]) & 0xFFFFFFFF)
    for rnd in range(10):
        if rnd > 0:                       # key schedule: bumped between rounds
            k0 = (k0 + _W0) & _MASK
            k1 = (k1 + _W1) & _MASK
        p0 = _M0 * c0                     # 32x32 -> 64 bit products
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    out = np.stack([c0, c1, c2, c3], axis=-1)
    return out.astype(np.uint32)


def philox_groups(seed, first_group, n_groups, stream=0):
    """Raw uint32 outputs (n_groups, 4) for groups first_group .. +n_groups-1."""
    g = np.arange(first_group, first_group + n_groups, dtype=np.uint64)
    ctr = np.empty((n_groups, 4), dtype=np.uint64)
    ctr[:, 0] = g & _MASK
    ctr[:, 1] = g >> _S32
    ctr[:, 2] = np.uint64(stream)
    ctr[:, 3] = 0
    seed = int(seed)
    return philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))


def uniforms(x, dtype):
    """Open-interval uniforms from raw outputs x (G, 4): (G, 4) for fp32, (G, 2) for fp64."""
    x = x.astype(np.uint64)
    if np.dtype(dtype) == np.float32:
        return ((x >> np.uint64(8)).astype(np.float64) + 0.5) * 2.0 ** -24
    a = ((x[:, 0] << _S32) | x[:, 1]) >> np.uint64(12)
    b = ((x[:, 2] << _S32) | x[:, 3]) >> np.uint64(12)
    return np.stack([(a.astype(np.float64) + 0.5) * 2.0 ** -52,
                     (b.astype(np.float64) + 0.5) * 2.0 ** -52], axis=-1)


def box_muller(u, v):
    r = np.sqrt(-2.0 * np.log(u))
    t = TWO_PI * v
    return r * np.cos(t), r * np.sin(t)


def philox_normal(seed, n, l, dtype, stream=0, chunk=1 << 22):
    """Omega (n x l) of iid N(0,1) in `dtype`, row-major element order."""
    dtype = np.dtype(dtype)
    per = 4 if dtype == np.float32 else 2
    total = int(n) * int(l)
    n_groups = (total + per - 1) // per
    flat = np.empty(n_groups * per, dtype=dtype)
    for g0 in range(0, n_groups, chunk):
        ng = min(chunk, n_groups - g0)
        u = uniforms(philox_groups(seed, g0, ng, stream), dtype)
        z = np.empty((ng, per), dtype=np.float64)
        z[:, 0], z[:, 1] = box_muller(u[:, 0], u[:, 1])
        if per == 4:
            z[:, 2], z[:, 3] = box_muller(u[:, 2], u[:, 3])
        flat[g0 * per:(g0 + ng) * per] = z.reshape(-1).astype(dtype)
    return flat[:total].reshape(int(n), int(l))
