"""Pins for the oracle's position reassignment of rotary-embedded keys (Sec. 3.1: consecutive
position ids after compression).  Independent statements: complex multiplication, the
cos/sin-table + rotate-half formulation written with torch, the relative-position property of
rotary embeddings, composition of rotations, and norm preservation."""
import numpy as np
import pytest
import torch

import oracle


def rope_complex(x, pos, theta, rot):
    """Rotary embedding at absolute positions `pos` via complex numbers (numpy, fp64)."""
    x = np.asarray(x, dtype=np.float64)
    half = rot // 2
    freq = theta ** (-2.0 * np.arange(half) / rot)
    z = (x[:, :half] + 1j * x[:, half:rot]) * np.exp(1j * np.asarray(pos, dtype=np.float64)[:, None] * freq[None, :])
    out = x.copy()
    out[:, :half] = z.real
    out[:, half:rot] = z.imag
    return out


def rope_rotate_half(x, pos, theta):
    """The cos/sin-table formulation used by the half-split convention (torch, fp64)."""
    x = torch.as_tensor(np.asarray(x, dtype=np.float64))
    d = x.shape[1]
    inv_freq = 1.0 / (theta ** (torch.arange(0, d, 2, dtype=torch.float64) / d))
    ang = torch.as_tensor(np.asarray(pos, dtype=np.float64))[:, None] * inv_freq[None, :]
    emb = torch.cat([ang, ang], dim=1)
    rot = torch.cat([-x[:, d // 2:], x[:, :d // 2]], dim=1)
    return (x * emb.cos() + rot * emb.sin()).numpy()


@pytest.mark.parametrize("d,rot,theta", [(8, 8, 10000.0), (64, 64, 1e6), (128, 64, 10000.0), (16, 0, 100.0)])
def test_matches_complex_multiplication(d, rot, theta):
    rng = np.random.default_rng(d + rot)
    n = 40
    k = rng.standard_normal((n, d)).astype(np.float32)
    kept = np.sort(rng.choice(500, size=n, replace=False)).astype(np.int32)
    got = oracle.rerotate_keys(k, kept, theta, rot)
    delta = np.arange(n) - kept
    want = rope_complex(k, delta, theta, rot) if rot else k.astype(np.float64)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    if rot == d:
        np.testing.assert_allclose(got, rope_rotate_half(k, delta, theta), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(np.linalg.norm(got, axis=1), np.linalg.norm(k.astype(np.float64), axis=1), rtol=1e-13)


def test_unmoved_rows_are_returned_bit_for_bit():
    rng = np.random.default_rng(3)
    k = rng.standard_normal((10, 16)).astype(np.float32)
    kept = np.array([0, 1, 2, 3, 9, 11, 12, 20, 21, 30], np.int32)
    got = oracle.rerotate_keys(k, kept)
    assert np.array_equal(got[:4], k[:4].astype(np.float64))
    assert not np.array_equal(got[4:], k[4:].astype(np.float64))


def test_reassigned_keys_are_the_original_keys_embedded_at_their_new_positions():
    """Embed un-rotated keys at their old positions, compact, re-rotate: the result equals
    embedding the same keys directly at positions 0..n-1.  With queries embedded at their own
    positions, the logits then depend only on the new relative distances."""
    rng = np.random.default_rng(4)
    d, theta, n = 32, 10000.0, 25
    raw = rng.standard_normal((n, d)).astype(np.float32)
    kept = np.sort(rng.choice(300, size=n, replace=False)).astype(np.int32)
    at_old = rope_complex(raw, kept, theta, d).astype(np.float32)       # what the cache holds (fp32 here)
    got = oracle.rerotate_keys(at_old, kept, theta)
    want = rope_complex(raw, np.arange(n), theta, d)
    np.testing.assert_allclose(got, want, rtol=0, atol=5e-6)             # only the fp32 storage of at_old
    raw_q = rng.standard_normal((1, d))
    logits = got @ rope_complex(raw_q, [n + 7], theta, d)[0]
    shifted = rope_complex(raw, np.arange(n) + 1000, theta, d) @ rope_complex(raw_q, [n + 7 + 1000], theta, d)[0]
    np.testing.assert_allclose(logits, shifted, rtol=0, atol=1e-4)       # relative-position property


def test_two_compactions_compose():
    rng = np.random.default_rng(5)
    d, theta = 16, 500.0
    k = rng.standard_normal((6, d)).astype(np.float32)
    first = np.array([2, 5, 6, 9, 10, 14], np.int32)          # slots 0..5 after the first compaction
    a = oracle.rerotate_keys(k, first, theta)
    second = np.array([0, 2, 3, 5], np.int32)                  # of those, these survive the next one
    b = oracle.rerotate_keys(a[second].astype(np.float32), second, theta)
    direct = oracle.rerotate_keys(k[second], first[second], theta)      # old slot -> final slot in one go
    np.testing.assert_allclose(b, direct, rtol=0, atol=2e-6)            # a is stored in fp32 in between


def test_bad_arguments():
    k = np.zeros((3, 8), np.float32)
    with pytest.raises(ValueError):
        oracle.rerotate_keys(k, np.arange(3), rot=3)
    with pytest.raises(ValueError):
        oracle.rerotate_keys(k, np.arange(3), rot=10)
    with pytest.raises(ValueError):
        oracle.rerotate_keys(k, np.arange(3), theta=0.0)
