"""Pins for the numpy statement of the blocked layouts (index identities of Fig. 4)."""
import numpy as np
import pytest

from oracle import layout


def test_activation_blocking_index_identity():
    N, C, H, W = 2, 35, 3, 4
    x = np.arange(N * C * H * W, dtype=np.float32).reshape(N, C, H, W)
    blk = layout.act_to_blocked(x)
    assert blk.shape == (N, 3, H, W, 16)
    flat = blk.ravel()
    for n, c, h, w in [(0, 0, 0, 0), (1, 34, 2, 3), (0, 16, 1, 2), (1, 15, 0, 3), (0, 31, 2, 0)]:
        off = (((n * 3 + c // 16) * H + h) * W + w) * 16 + c % 16      # input[img][ifm_tile][ij][ii][ifm]
        assert flat[off] == x[n, c, h, w]
    # pad lanes (channels 35..47) are +0.0, bit pattern included
    assert not blk[:, 2, :, :, 3:].view(np.uint32).any()
    np.testing.assert_array_equal(layout.blocked_to_act(blk, C), x)


def test_filter_blocking_index_identity():
    K, C, R, S = 32, 20, 3, 2
    w = np.arange(K * C * R * S, dtype=np.float32).reshape(K, C, R, S)
    blk = layout.filt_to_blocked(w)
    assert blk.shape == (2, 2, R, S, 16, 16)
    flat = blk.ravel()
    for k, c, r, s in [(0, 0, 0, 0), (31, 19, 2, 1), (16, 3, 1, 0), (15, 16, 0, 1), (17, 1, 2, 0)]:
        # filter[ofm_tile][ifm_tile][kj][ki][ifm][ofm]: ofm fastest, then ifm
        off = (((((k // 16) * 2 + c // 16) * R + r) * S + s) * 16 + c % 16) * 16 + k % 16
        assert flat[off] == w[k, c, r, s]
    assert not blk[:, 1, :, :, 4:, :].view(np.uint32).any()
    np.testing.assert_array_equal(layout.blocked_to_filt(blk, C), w)


def test_output_blocking_roundtrip_and_rejects_ragged_k():
    y = np.random.default_rng(0).standard_normal((2, 48, 3, 5))
    blk = layout.out_to_blocked(y)
    assert blk.shape == (2, 3, 3, 5, 16)
    assert blk[1, 2, 1, 4, 7] == y[1, 39, 1, 4]
    np.testing.assert_array_equal(layout.blocked_to_out(blk), y)
    with pytest.raises(ValueError):
        layout.out_to_blocked(np.zeros((1, 20, 2, 2)))
    with pytest.raises(ValueError):
        layout.filt_to_blocked(np.zeros((20, 16, 1, 1)))


def test_bit_patterns_survive(capsys):
    # NaN payloads, infinities and negative zero must move unchanged
    bits = np.array([0x7FC00001, 0xFFC12345, 0x7F800000, 0xFF800000, 0x80000000, 0x00000001], np.uint32)
    x = np.resize(bits, (1, 6, 1, 2)).view(np.float32)
    back = layout.blocked_to_act(layout.act_to_blocked(x), 6)
    np.testing.assert_array_equal(back.view(np.uint32), x.view(np.uint32))


def test_packed8_filter_layout_is_a_permutation_of_the_standard_one():
    K, C, R, S = 32, 20, 3, 2
    w = np.arange(K * C * R * S, dtype=np.uint16).reshape(K, C, R, S)
    std = layout.filt_to_blocked(w)
    p8 = layout.filt_to_blocked_packed8(w)
    assert p8.shape == (2, 2, R, S, 2, 16, 8)
    flat = p8.ravel()
    for k, c, r, s in [(0, 0, 0, 0), (31, 19, 2, 1), (16, 3, 1, 0), (15, 16, 0, 1), (17, 9, 2, 0), (5, 8, 1, 1)]:
        cc, kk = c % 16, k % 16
        off = ((((((k // 16) * 2 + c // 16) * R + r) * S + s) * 2 + cc // 8) * 16 + kk) * 8 + cc % 8
        assert flat[off] == w[k, c, r, s]
    # same multiset per block, zero lanes included
    assert np.array_equal(np.sort(p8.reshape(2, 2, R, S, 256), -1), np.sort(std.reshape(2, 2, R, S, 256), -1))
    np.testing.assert_array_equal(layout.blocked_packed8_to_filt(p8, C), w)
