"""The seeded input streams (NumPy side): the Philox rounds against an arbitrary-precision
integer restatement, sample moments, and random access == contiguous fill.  CPU only.
The published known-answer vectors of Philox are not in this container, so the round
function is pinned by two independently written forms and by its statistics; parity of the
gradient path never depends on it (both sides consume the same numbers)."""
import numpy as np

from paper_2605_11215_amd.synth import reference_np as S


def philox_int(ctr, key):
    """Philox4x32-10 on Python integers, written from the SC'11 description."""
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        hi0, lo0 = divmod(0xD2511F53 * c[0], 1 << 32)
        hi1, lo1 = divmod(0xCD9E8D57 * c[2], 1 << 32)
        c = [hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0]
        k = [(k[0] + 0x9E3779B9) % (1 << 32), (k[1] + 0xBB67AE85) % (1 << 32)]
    return c


def test_round_function_two_forms_agree():
    rng = np.random.default_rng(1)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 1 << 32, 4)]
        key = [int(x) for x in rng.integers(0, 1 << 32, 2)]
        got = [int(np.asarray(w).reshape(-1)[0]) for w in S.philox4x32_10(*ctr, *key)]
        assert got == philox_int(ctr, key)
    # bijection on the counter for a fixed key: distinct counters give distinct outputs
    x = S.philox4x32_10(np.arange(1 << 16), 5, 6, 7, 1, 0)
    packed = (x[0] << np.uint64(32)) | x[1]
    assert len(np.unique(packed)) == 1 << 16


def test_normal_stream_moments_and_independence():
    x = S.fill(1 << 21, 1, S.TAG_GRAD, 3, 1, 1.0).astype(np.float64)
    n = len(x)
    assert abs(x.mean()) < 4 / np.sqrt(n)
    assert abs(x.std() - 1) < 4 / np.sqrt(2 * n)
    assert abs((x ** 3).mean()) < 4 * np.sqrt(15 / n)
    assert abs((x ** 4).mean() - 3) < 4 * np.sqrt(96 / n)
    assert abs(np.corrcoef(x[:-1], x[1:])[0, 1]) < 4 / np.sqrt(n)
    y = S.fill(1 << 21, 1, S.TAG_GRAD, 4, 1, 1.0).astype(np.float64)       # next microbatch
    assert abs(np.corrcoef(x, y)[0, 1]) < 4 / np.sqrt(n)
    z = S.fill(1 << 21, 1, S.TAG_GRAD, 3, 2, 1.0).astype(np.float64)       # next iteration
    assert abs(np.corrcoef(x, z)[0, 1]) < 4 / np.sqrt(n)
    s = S.fill(1 << 16, 1, S.TAG_GRAD, 3, 1, 1e-3)
    assert np.array_equal(s, (1e-3 * x[:1 << 16] / 1.0).astype(np.float32)) or \
        np.max(np.abs(s / 1e-3 - x[:1 << 16])) < 1e-6


def test_student_t3_stream():
    t = S.fill(1 << 20, 7, S.TAG_GRAD, 0, 0, 1.0, kind=S.KIND_STUDENT_T3).astype(np.float64)
    # quartiles of Student-t with 3 degrees of freedom: +-0.7649; P(|t| > 3.182) = 0.05
    assert abs(np.quantile(t, 0.75) - 0.7649) < 0.01 and abs(np.quantile(t, 0.25) + 0.7649) < 0.01
    assert abs((np.abs(t) > 3.182).mean() - 0.05) < 0.002
    assert np.abs(t).max() > 30                                             # heavy tail


def test_random_access_equals_contiguous_fill():
    idx = np.arange(5, 100003, dtype=np.uint64)
    for kind in (S.KIND_NORMAL, S.KIND_STUDENT_T3):
        a = S.values(idx, 1, 0, 3, 1, 1e-3, kind)
        b = S.fill(len(idx), 1, 0, 3, 1, 1e-3, kind, start=5)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    big = np.array([0, 3, (1 << 31) + 5, 1978662911], np.uint64)            # past 2**31
    assert np.all(np.isfinite(S.values(big, 1, 0, 0, 0, 1e-3)))


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e-5, 0.0, -0.0], np.float32)
    # 1 + 2^-8 is a tie -> even (1.0); 1 + 3*2^-8 is a tie -> even (1 + 2^-6)
    h = S.f32_to_bf16_bits(x)
    back = S.bf16_bits_to_f32(h)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625) and back[3] == -1.0
    assert abs(back[4] - x[4]) <= abs(x[4]) * 2.0 ** -8
    assert h[5] == 0 and h[6] == 0x8000
    r = np.random.default_rng(0).normal(0, 1e-3, 10000).astype(np.float32)
    tb = torch_bf16(r)
    assert np.array_equal(S.bf16_bits_to_f32(S.f32_to_bf16_bits(r)), tb)


def torch_bf16(x):
    import torch
    return torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
