"""Counter-based factor generator of the oracle: Philox4x32-10 + Box-Muller.

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper only says that directions are regenerated from a seed when they are
consumed (Sec. 2.2, the MeZO row of the taxonomy table) and that U and V have
independent standard-normal entries (Sec. 3.3, appendix on the multivariate
CLT).  It names no generator.  The reading taken here is the published
Philox4x32-10 bijection (Salmon, Moraes, Dror, Shaw, SC'11) followed by the
textbook Box-Muller transform.

Pins
  * philox4x32_10: the known-answer vectors published with the algorithm
    (tests/golden/philox4x32_10_kat.txt).
  * normals: closed-form moments, the hard |z| bound implied by u >= 2^-24,
    a Kolmogorov-Smirnov test against the normal CDF, and the entry statistics
    of U V^T / sqrt(r) from the CLT appendix (variance 1, excess kurtosis 6/r).
  * the counter / lane layout (which word feeds which matrix entry) is this
    build's own definition: "parity unpinned" by the paper; it is pinned only by
    a brute-force scalar re-derivation on tiny shapes and by bit-equality of the
    two implementations.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint64(0x9E3779B9)
_W1 = np.uint64(0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(counter, key):
    """Philox4x32 with 10 rounds.

    counter: integer array [..., 4], key: integer array [..., 2] (broadcast
    against each other on the leading axes); every entry is a 32-bit word.
    Returns uint32 array [..., 4].

    One round maps (c0, c1, c2, c3) to
        (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0))
    and the key is advanced by the two Weyl constants between rounds.
    """
    counter = np.asarray(counter).astype(np.uint64)
    key = np.asarray(key).astype(np.uint64)
    lead = np.broadcast_shapes(counter.shape[:-1], key.shape[:-1])
    c = [np.broadcast_to(counter[..., i], lead).copy() for i in range(4)]
    k = [np.broadcast_to(key[..., i], lead).copy() for i in range(2)]
    for rnd in range(10):
        if rnd > 0:
            k[0] = (k[0] + _W0) & _MASK
            k[1] = (k[1] + _W1) & _MASK
        p0 = _M0 * c[0]
        p1 = _M1 * c[2]
        c = [(p1 >> _S32) ^ c[1] ^ k[0], p1 & _MASK,
             (p0 >> _S32) ^ c[3] ^ k[1], p0 & _MASK]
    return np.stack(c, axis=-1).astype(np.uint32)


def factor_words(seed, tensor_id, n_blocks, first_block=0):
    """Raw words of the factor stream: block q uses counter
    (q mod 2^32, q div 2^32, tensor_id, 0) and key (seed mod 2^32, seed div 2^32).
    Returns uint32 [n_blocks, 4]."""
    seed = int(seed)
    q = np.arange(first_block, first_block + n_blocks, dtype=np.uint64)
    ctr = np.stack([q & _MASK, q >> _S32,
                    np.full_like(q, int(tensor_id) & 0xFFFFFFFF),
                    np.zeros_like(q)], axis=-1)
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint64)
    return philox4x32_10(ctr, key)


def uniform_open01(words):
    """u(w) = (2*(w >> 9) + 1) * 2^-24: 2^23 equally spaced points strictly
    inside (0, 1), each exactly representable in fp32 (and in fp64)."""
    w = np.asarray(words).astype(np.uint64)
    return ((w >> np.uint64(9)) * np.uint64(2) + np.uint64(1)).astype(np.float64) * 2.0 ** -24


def normals_from_words(words):
    """Box-Muller on word pairs: words [..., 4] -> normals [..., 4] (fp64).
    (w0, w1) gives entries 0 and 1, (w2, w3) gives entries 2 and 3:
        rho = sqrt(-2 ln u(w_a));  z_first = rho cos(2 pi u(w_b));  z_second = rho sin(2 pi u(w_b))
    """
    u = uniform_open01(words)
    out = np.empty(u.shape, dtype=np.float64)
    for a in (0, 2):
        rho = np.sqrt(-2.0 * np.log(u[..., a]))
        ang = 2.0 * np.pi * u[..., a + 1]
        out[..., a] = rho * np.cos(ang)
        out[..., a + 1] = rho * np.sin(ang)
    return out


def round_to_bf16(x):
    """Round fp32 values to the nearest bfloat16 (ties to even); result is
    returned as fp32 holding exactly representable bf16 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = rounded.astype(np.uint32).view(np.float32).reshape(x.shape)
    nan = np.isnan(x)
    if nan.any():
        out = out.copy()
        out[nan] = np.nan
    return out


def factor_matrix(seed, tensor_id, rows, r, dtype="f32"):
    """Factor matrix [rows, r] of i.i.d. N(0,1) entries (Sec. 3.3).

    Entry (i, j) has flat index e = i*r + j and is entry (e mod 4) of block
    e div 4 of the stream (seed, tensor_id).  The fp64 Box-Muller value is
    rounded once to fp32; with dtype "bf16" it is then rounded to bf16 (the
    value every consumer of the factor sees in the bf16 configurations).
    Returns fp64 array holding those rounded values.
    """
    n = rows * r
    n_blocks = (n + 3) // 4
    z = normals_from_words(factor_words(seed, tensor_id, n_blocks)).reshape(-1)[:n]
    z32 = z.astype(np.float32)
    if dtype == "bf16":
        z32 = round_to_bf16(z32)
    elif dtype != "f32":
        raise ValueError(dtype)
    return z32.astype(np.float64).reshape(rows, r)


def u_tensor_id(tensor_id):
    """Stream id of U for a layer whose (even) tensor id is given."""
    return int(tensor_id) & ~1


def v_tensor_id(tensor_id):
    """Stream id of V: the odd neighbour of the layer's even tensor id."""
    return int(tensor_id) | 1
