"""Counter-based noise for the oracle (test infrastructure, never product code).

The paper only requires xi, eta ~ N(0, I), i.i.d. across nodes, steps and
latent elements (Eq. 2; App. B.1 "fresh draws at each split, no cross-time
sharing").  To let two independent implementations draw the *same* numbers the
workloads fix a counter-based generator: Philox4x32 with 10 rounds as defined
by Salmon, Moraes, Dror and Shaw, "Parallel random numbers: as easy as 1, 2,
3" (SC'11), keyed by the 64-bit seed, with the counter naming (element quad,
node id, step, stream).

Pins (tests/test_oracle_philox.py): the raw words reproduce the generator's
published known-answer vectors (all-zero, all-ones and pi-digit counter and
key; tests/golden/philox4x32_10_known_answers.txt); the round function is a
bijection with the inverse written from the definition; the normals pass
moment, KS and independence checks; sibling covariance is 1/(1+s^2) (App. B.1).
"""
import numpy as np

# Multipliers and Weyl key increments of Philox4x32 (SC'11, Table 2 / Sec. 3.3).
_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)

# Stream tags (4th counter word).
TAG_ETA = 0    # per-child innovation eta_b (node id = child)
TAG_XI0 = 1    # shared component xi_0 of a split (node id = parent)
TAG_ROOT = 2   # root latent z_0 (node id = noise group, step 0)
TAG_DEPTH = 3  # seeded depth-pruning subset


def philox_round(c, k0, k1):
    """One Philox4x32 round on counters c [..., 4] (uint64 holding 32-bit words)."""
    p0 = _M0 * c[..., 0]
    p1 = _M1 * c[..., 2]
    hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
    hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
    out = np.empty_like(c)
    out[..., 0] = hi1 ^ c[..., 1] ^ np.uint64(k0)
    out[..., 1] = lo1
    out[..., 2] = hi0 ^ c[..., 3] ^ np.uint64(k1)
    out[..., 3] = lo0
    return out


def philox4x32_10(counter, seed):
    """Ten rounds; key = (low 32 bits of seed, high 32 bits), bumped by the Weyl
    constants between rounds.  counter: integer array [..., 4] -> uint32 [..., 4]."""
    c = np.asarray(counter).astype(np.uint64) & _MASK32
    k0 = int(seed) & 0xFFFFFFFF
    k1 = (int(seed) >> 32) & 0xFFFFFFFF
    for r in range(10):
        c = philox_round(c, k0, k1)
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return c.astype(np.uint32)


def words(seed, node_id, step, tag, n_quads):
    """Raw words of one stream: [n_quads, 4] uint32, counter = (q, node, step, tag)."""
    ctr = np.empty((n_quads, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(n_quads, dtype=np.uint64)
    ctr[:, 1] = np.uint64(int(node_id) & 0xFFFFFFFF)
    ctr[:, 2] = np.uint64(int(step) & 0xFFFFFFFF)
    ctr[:, 3] = np.uint64(int(tag) & 0xFFFFFFFF)
    return philox4x32_10(ctr, seed)


def uniform(x):
    """32-bit word -> u in (0, 1): the top 23 bits, centred in their cell, so
    that u = (2k+1) / 2^24 is exactly representable in fp32 as well."""
    return ((np.asarray(x, dtype=np.uint32) >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def normals(seed, node_id, step, tag, D):
    """D standard normals (fp64) of one stream.  Element e uses word e%4 of quad
    e//4; Box-Muller on the word pairs (0,1) and (2,3): the first word gives the
    radius, the second the angle; cos goes to the even element, sin to the odd."""
    assert D % 4 == 0
    w = words(seed, node_id, step, tag, D // 4)
    u = uniform(w)
    out = np.empty((D // 4, 4), dtype=np.float64)
    for a, b in ((0, 1), (2, 3)):
        r = np.sqrt(-2.0 * np.log(u[:, a]))
        th = 2.0 * np.pi * u[:, b]
        out[:, a] = r * np.cos(th)
        out[:, b] = r * np.sin(th)
    return out.reshape(D)
