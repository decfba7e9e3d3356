"""The seeded generators: reproducible, counter-based, right moments, exactly
representable in the storage type (no GPU)."""
import numpy as np

from workload import gen


def test_uniform_is_counter_based_and_in_range():
    a = gen.uniform01(5, 7, 1000)
    assert (a >= 0).all() and (a < 1).all()
    assert np.array_equal(a[100:200], gen.uniform01(5, 7, 100, offset=100))
    assert not np.array_equal(a, gen.uniform01(6, 7, 1000))
    assert not np.array_equal(a, gen.uniform01(5, 8, 1000))
    # a fixed value so that another implementation can check its generator
    z = gen.uniform01(0, 0, 1)[0]
    assert 0.0 <= z < 1.0 and z == gen.uniform01(0, 0, 3)[0]


def test_normal_moments():
    v = gen.normal(1, 2, 400_000)
    assert abs(v.mean()) < 0.01 and abs(v.std() - 1) < 0.01
    assert abs((v ** 3).mean()) < 0.03 and abs((v ** 4).mean() - 3) < 0.1


def test_bf16_rounding_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 0.0], np.float32)
    q = gen.quantize(x, "bf16")
    assert list(q) == [1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -2.5, 0.0]
    r = gen.normal(0, 0, 1000).astype(np.float32)
    assert np.abs(gen.quantize(r, "bf16") - r).max() <= 2 ** -8 * np.abs(r).max()


def test_model_tensors_and_blob_layout():
    shapes = [(4, 3, 3, 3), (5, 4, 1, 1), (7, 5, 1, 1)]
    w, b = gen.model_tensors(shapes, seed=9)
    for t, s in zip(w, shapes):
        assert t.shape == s and t.dtype == np.float32
        assert np.array_equal(t.astype(np.float16).astype(np.float32), t)
    blob = gen.pack_blob(w, b)
    assert blob.size == gen.blob_bytes(shapes)
    nw = sum(int(np.prod(s)) for s in shapes)            # 108+20+35 = 163 (odd -> pad)
    halves = blob[:2 * nw].view(np.float16).astype(np.float32)
    assert np.array_equal(halves, np.concatenate([t.ravel() for t in w]))
    off = 2 * nw + (-2 * nw) % 4
    assert np.array_equal(blob[off:].view(np.float32), np.concatenate(b))
    big, _ = gen.model_tensors([(64, 512, 3, 3)], seed=1)
    assert abs(big[0].std() - np.sqrt(2 / (512 * 9))) < 0.02 * np.sqrt(2 / (512 * 9))
    _, bb = gen.model_tensors([(20000, 1, 1, 1)], seed=1)
    assert abs(bb[0].std() - 0.1) < 0.003


def test_images_do_not_depend_on_batch_cut():
    a = gen.images(4, 0, 4, 3, 8, 8)
    b = gen.images(4, 2, 2, 3, 8, 8)
    assert np.array_equal(a[2:], b)
    u = gen.images(4, 0, 2, 3, 16, 16, "uniform")
    assert u.min() >= -1 and u.max() <= 1
    assert np.array_equal(u.astype(np.float16).astype(np.float32), u)
