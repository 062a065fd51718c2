"""Pins for the oracle's wire form of the (blockwise) scaled-sign message."""
import numpy as np


def test_pack_is_numpy_packbits_little_endian(oracle):
    rng = np.random.default_rng(0)
    for d in (1, 7, 8, 9, 1000, 4099):
        v = rng.standard_normal(d).astype(np.float32)
        v[::5] = 0.0
        v[1::7] = -0.0
        got = oracle.pack_sign(v)
        assert np.array_equal(got, np.packbits(v < 0, bitorder="little"))
        assert got.size == (d + 7) // 8          # one bit per element: the 32x the paper quotes


def test_unpack_inverts_pack_into_the_compressed_message(oracle):
    rng = np.random.default_rng(1)
    v = rng.standard_normal(3001).astype(np.float32)
    p, desc = oracle.compress("sign", v)
    assert np.array_equal(oracle.unpack_sign(oracle.pack_sign(v), v.size, desc.scale), p)
    off = [0, 5, 1000, 1001, 3001]
    pb, scales = oracle.compress_blocksign(v, off)
    assert np.array_equal(oracle.unpack_sign(oracle.pack_sign(v), v.size, scales, off), pb)
