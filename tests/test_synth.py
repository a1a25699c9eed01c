"""The seeded input generator: deterministic, sliceable, N(0,1)-shaped, integer-only."""
import numpy as np
import torch

from paper_2502_12574_amd import synth


def test_slices_regenerate_bit_exactly():
    full = synth.draw_k(7, 1, 3, 0, 4096)
    for a, n in ((0, 1), (17, 100), (4000, 96)):
        assert torch.equal(synth.draw_k(7, 1, 3, a, n), full[a:a + n])
    assert synth.draw_v(7, 1, 3, 5, 0).shape == (0, 128)
    far = synth.draw_v(7, 0, 0, (1 << 22) - 8, 8)          # 4M-token contexts index beyond 2**31 bytes
    assert far.shape == (8, 128) and torch.isfinite(far.float()).all()


def test_streams_differ_by_every_key_field():
    base = synth.draw(1, synth.TENSOR_K, 0, 0, 0, 64)
    for args in ((2, synth.TENSOR_K, 0, 0), (1, synth.TENSOR_V, 0, 0), (1, synth.TENSOR_K, 1, 0),
                 (1, synth.TENSOR_K, 0, 1)):
        other = synth.draw(*args, 0, 64)
        assert (other != base).float().mean() > 0.9


def test_distribution_is_standard_normal():
    x = synth.draw_q(3, 0, 5, 0, 1 << 14).float().numpy().ravel()
    assert abs(x.mean()) < 5e-3 and abs(x.std() - 1.0) < 5e-3
    assert abs(np.mean(x ** 3)) < 2e-2 and abs(np.mean(x ** 4) - 3.0) < 5e-2
    m = x.reshape(-1, 128)
    assert abs(np.mean(m[:-1] * m[1:])) < 5e-3 and abs(np.mean(m[:, :-1] * m[:, 1:])) < 5e-3
    t = synth.normal_table().float()
    assert t.shape == (65536,) and torch.all(t[1:] >= t[:-1]) and torch.equal(t, -t.flip(0))


def test_peaked_keys():
    k = synth.draw_k(9, 0, 2, 0, 20000).float()
    kp = synth.draw_k(9, 0, 2, 0, 20000, peaked=True).float()
    m = synth.peaked_key_mask(9, 0, 2, 0, 20000)
    assert 0.08 < m.float().mean() < 0.12
    assert torch.equal(kp[m], 4 * k[m]) and torch.equal(kp[~m], k[~m])
