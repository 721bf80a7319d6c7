"""Counter-based random numbers for the oracle (test infrastructure only).

The paper only says that the initial latents and the per-step noise are
standard normal (Sec. 5.1, the sentence introducing the group of G latents and
the Euler-Maruyama update).  The stream used here is Philox-4xW-10 of Salmon,
Moraes, Dror and Shaw, "Parallel random numbers: as easy as 1, 2, 3" (SC'11),
written from that paper's description of the round: two W x W -> 2W products,
an S-box-free permutation of the four words, and a Weyl key schedule.

Pins
----
* ``philox4_scalar`` is generic in the word width.  Its W=64 instance is
  compared with ``numpy.random.Philox`` (an independent implementation of
  Philox-4x64-10), which fixes the round structure, the word permutation, the
  key schedule and the round count.
* ``philox4x32`` (vectorised, W=32) is compared with ``philox4_scalar(W=32)``.
* The W=32 multipliers / Weyl increments: the two increments have a closed form (fractional parts of
  the golden ratio and of sqrt(3) - 1, truncated to the word), checked in exact integer arithmetic; all
  four are compared with the values the GPU vendor's random-number library states in its installed
  header, and the whole W=32 block function with that library's own generator (a known-answer test that
  runs where the library can allocate, i.e. next to a GPU).
* ``normals`` is checked by moments and a Kolmogorov-Smirnov test.
"""
import numpy as np

# word-width specific constants of Philox-4xW (SC'11 paper, Table of constants)
_CONST = {
    32: dict(M0=0xD2511F53, M1=0xCD9E8D57, W0=0x9E3779B9, W1=0xBB67AE85),
    64: dict(M0=0xD2E7470EE14C6C93, M1=0xCA5A826395121157,
             W0=0x9E3779B97F4A7C15, W1=0xBB67AE8584CAA73B),
}

# stream tags: fourth counter word
STREAM_INIT = 0      # initial latents x_0 ~ N(0, I)
STREAM_STEP = 1      # per-step noise xi of the Euler-Maruyama update


def philox4_scalar(counter, key, W=32, rounds=10):
    """One Philox-4xW block on Python integers. counter: 4 words, key: 2 words."""
    c = _CONST[W]
    mask = (1 << W) - 1
    x0, x1, x2, x3 = [int(v) & mask for v in counter]
    k0, k1 = [int(v) & mask for v in key]
    for r in range(rounds):
        if r > 0:                      # Weyl sequence on the key between rounds
            k0 = (k0 + c["W0"]) & mask
            k1 = (k1 + c["W1"]) & mask
        p0 = c["M0"] * x0              # full 2W-bit products
        p1 = c["M1"] * x2
        hi0, lo0 = p0 >> W, p0 & mask
        hi1, lo1 = p1 >> W, p1 & mask
        x0, x1, x2, x3 = hi1 ^ x1 ^ k0, lo1, hi0 ^ x3 ^ k1, lo0
    return (x0, x1, x2, x3)


def philox4x32(c0, c1, c2, c3, k0, k1, rounds=10):
    """Vectorised Philox-4x32-10. All arguments broadcastable uint arrays / ints.

    Returns four uint32 arrays."""
    c = _CONST[32]
    m32 = np.uint64(0xFFFFFFFF)
    sh = np.uint64(32)
    x0, x1, x2, x3 = np.broadcast_arrays(*[np.asarray(v, dtype=np.uint64) & m32
                                           for v in (c0, c1, c2, c3)])
    k0 = np.uint64(int(k0) & 0xFFFFFFFF)
    k1 = np.uint64(int(k1) & 0xFFFFFFFF)
    M0, M1 = np.uint64(c["M0"]), np.uint64(c["M1"])
    W0, W1 = np.uint64(c["W0"]), np.uint64(c["W1"])
    for r in range(rounds):
        if r > 0:
            k0 = (k0 + W0) & m32
            k1 = (k1 + W1) & m32
        p0 = M0 * x0                  # < 2^64, no overflow
        p1 = M1 * x2
        hi0, lo0 = p0 >> sh, p0 & m32
        hi1, lo1 = p1 >> sh, p1 & m32
        x0, x1, x2, x3 = hi1 ^ x1 ^ k0, lo1, hi0 ^ x3 ^ k1, lo0
    return tuple(v.astype(np.uint32) for v in (x0, x1, x2, x3))


def uint32_words(seed, stream, orig_id, step, n_elem):
    """The raw 32-bit stream for one trajectory: word e of the result is output
    (e mod 4) of the block with counter (e div 4, step, orig_id, stream) and key
    (seed low word, seed high word)."""
    nblk = (n_elem + 3) // 4
    blk = np.arange(nblk, dtype=np.uint64)
    w = philox4x32(blk, step, orig_id, stream, seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return np.stack(w, axis=1).reshape(-1)[:n_elem]


def normals(seed, stream, orig_id, step, n_elem):
    """n_elem standard normals (fp64) for trajectory ``orig_id`` at ``step``.

    Each Philox block (n0, n1, n2, n3) gives four normals by the Box-Muller
    transform on the pairs (n0, n1) and (n2, n3):
        u_a = (n_a + 1/2) / 2^32  in (0, 1)
        z   = sqrt(-2 ln u_a) * (cos 2 pi u_b, sin 2 pi u_b).
    Element e of the trajectory takes normal (e mod 4) of block (e div 4).
    Keyed by the trajectory's ORIGINAL id, so pruning never changes the noise a
    surviving trajectory sees."""
    nblk = (n_elem + 3) // 4
    w = uint32_words(seed, stream, orig_id, step, 4 * nblk).reshape(nblk, 4).astype(np.float64)
    u = (w + 0.5) / 4294967296.0
    out = np.empty((nblk, 4), dtype=np.float64)
    for a, b in ((0, 1), (2, 3)):
        r = np.sqrt(-2.0 * np.log(u[:, a]))
        ang = 2.0 * np.pi * u[:, b]
        out[:, a] = r * np.cos(ang)
        out[:, b] = r * np.sin(ang)
    return out.reshape(-1)[:n_elem]
