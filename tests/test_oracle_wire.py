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


def test_topk_message_lists_the_kept_entries_in_index_order(oracle):
    rng = np.random.default_rng(2)
    for d, k in ((1, 1), (40, 7), (64, 64), (5000, 123)):
        v = rng.choice(np.array([0.0, -0.0, 0.5, -0.5, 1.0, 2.0, -2.0], dtype=np.float32), size=d)
        m = rng.random(d) < 0.5
        v[m] = rng.standard_normal(m.sum()).astype(np.float32)
        idx, val = oracle.pack_topk(v, k)
        assert idx.size == k and np.all(np.diff(idx.astype(np.int64)) > 0)         # 8k bytes, ascending, distinct
        assert np.array_equal(val.view(np.uint32), v[idx].view(np.uint32))
        brute = sorted(sorted(range(d), key=lambda j: (-abs(float(v[j])), j))[:k])  # Definition 2, ties to lower index
        assert idx.tolist() == brute
        p, _ = oracle.compress("topk", v, k)
        assert np.array_equal(oracle.unpack_topk(idx, val, d).view(np.uint32), p.view(np.uint32))
